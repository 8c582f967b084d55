// Device-side building blocks shared by the gfx950 kernels of the Quartet MXFP4 path.
// Internal to the HIP library (not part of the C ABI, not used by the CPU oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quartet {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kGroup = 32;                      // Hadamard block = MX group (Section 4.4)
constexpr float kInvSqrt32 = 0.17677669529663687f;  // fl(1/sqrt 32) = 0x3E3504F3

enum QuantMode { kFwd = 0, kBwdRtn = 1, kBwdSr = 2 };

// Byte offset of the E8M0 scale of (row, group g = k/32) in the tiled scale layout: tiles of
// 32 rows x 8 groups (256 K-elements), 256 bytes each, ordered [row block][K-quad]; inside a tile
// byte ((g&1)*32 + row%32)*4 + (g%8)/2.  Lane l of a wave that owns a 32-row block of an MFMA
// operand therefore finds its four K=64-step scales in dword l of the tile.  kq = ceil(k/256).
__host__ __device__ __forceinline__ uint64_t scale_tile_offset(uint32_t row, uint32_t g, uint32_t kq) {
    return ((uint64_t)(row >> 5) * kq + (g >> 3)) * 256u + (((g & 1u) << 5) + (row & 31u)) * 4u + ((g & 7u) >> 1);
}

// n / d for n < 2^31 by multiply-high with a host-computed magic number (Granlund-Montgomery).
struct FastDiv {
    uint32_t mul, shift;
};
__device__ __forceinline__ uint32_t fast_div(uint32_t n, FastDiv f) { return (__umulhi(n, f.mul) + n) >> f.shift; }

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// Five butterfly stages of the 32-point Walsh-Hadamard transform in natural (Sylvester) order,
// stride 1,2,4,8,16, then the normalization multiply (Section 3, "Outlier mitigation").  Each
// stage is a separate fp32 add/sub: the build disables FMA contraction.
__device__ __forceinline__ void fwht32(float (&v)[32]) {
#pragma unroll
    for (int h = 1; h < 32; h <<= 1) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            if ((i & h) == 0) {
                float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = v[i] * kInvSqrt32;
}

// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> four 32-bit words.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Stochastic rounding of v (|v| < 6) onto the E2M1 grid with a 16-bit draw r (Section 3,
// "Rounding"): with lo <= |v| < hi adjacent grid points and f = (|v|-lo)/(hi-lo), the result is
// hi iff (r + 1/2) / 2^16 < f.  Returns the 4-bit code (bit 3 = sign bit of v).
//  |v| >= 1: the grid keeps one mantissa bit, f is the 22 discarded bits F / 2^22, and
//            f > (r + 1/2)/2^16  <=>  F >= 64 r + 33  <=>  F + 2^22 - 64 r - 33 carries into bit 22.
//  |v| <  1: the grid is {0, 1/2, 1}; with u = (r + 1/2)/2^16 the code is the number of the
//            thresholds u, 1 + u that 2|v| exceeds = ceil(fl(2|v| - u)); the subtraction's sign is
//            exact, and when 2|v| >= 1 both operands are multiples of 2^-23 below 2, so it is exact.
__device__ __forceinline__ uint32_t sr_e2m1(float v, uint32_t r) {
    uint32_t bits = f2u(v);
    uint32_t abits = bits & 0x7FFFFFFFu;
    // large path
    uint32_t t = abits + (0x400000u - 33u) - (r << 6);
    uint32_t code_large = (t >> 22) - 252u;
    // small path
    float u = u2f(0x3F800040u | (r << 7)) - 1.0f;          // (r + 1/2) / 2^16, exact
    float d = __builtin_fmaf(u2f(abits), 2.0f, -u);        // fl(2|v| - u): one rounding
    uint32_t code_small = (uint32_t)(int)__builtin_ceilf(d);
    uint32_t code = (abits >= 0x3F800000u) ? code_large : code_small;
    return code | ((bits >> 28) & 8u);
}

}  // namespace quartet
