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

typedef unsigned int v4u_t __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) 16-byte and 4-byte accesses for data that is touched once: measured
// 7.0 TB/s against 6.3 TB/s for plain loads on a read-only sweep of 2 GiB.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    v4u_t v = __builtin_nontemporal_load(static_cast<const v4u_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void* p, const uint4& q) {
    v4u_t v = {q.x, q.y, q.z, q.w};
    __builtin_nontemporal_store(v, static_cast<v4u_t*>(p));
}
__device__ __forceinline__ uint32_t load_stream4(const void* p) {
    return __builtin_nontemporal_load(static_cast<const uint32_t*>(p));
}
__device__ __forceinline__ void store_stream4(void* p, uint32_t v) {
    __builtin_nontemporal_store(v, static_cast<uint32_t*>(p));
}

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// Five butterfly stages of the 32-point Walsh-Hadamard transform in natural (Sylvester) order,
// stride 1,2,4,8,16 (Section 3, "Outlier mitigation").  Each stage is a separate fp32 add/sub: the
// build disables FMA contraction.  The normalization multiply is the caller's.
__device__ __forceinline__ void fwht32_unscaled(float (&v)[32]) {
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
}
__device__ __forceinline__ void fwht32(float (&v)[32]) {
    fwht32_unscaled(v);
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = v[i] * kInvSqrt32;
}

// Hadamard blocks of nb = 2, 4 or 8 groups (64, 128, 256 elements; Section 4.4, "Costs and format
// specialization"): H_{32 nb} = H_nb (x) H_32, evaluated as the butterflies that combine whole groups
// first (stride 32, 64, 128 elements), then fwht32_unscaled inside each group, then one multiply by
// fl(1/sqrt(32 nb)).
__device__ __forceinline__ float block_norm(uint32_t nb) {
    return nb == 1u ? kInvSqrt32 : nb == 2u ? 0.125f : nb == 4u ? 0.08838834764831845f /* fl(1/sqrt 128) */ : 0.0625f;
}

// value of lane (l ^ XOR), XOR = 1, 2 or 4
template <int XOR> __device__ __forceinline__ float lane_xor(float x);
template <> __device__ __forceinline__ float lane_xor<1>(float x) {
    return u2f((uint32_t)__builtin_amdgcn_update_dpp(0, (int)f2u(x), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true));
}
template <> __device__ __forceinline__ float lane_xor<2>(float x) {
    return u2f((uint32_t)__builtin_amdgcn_update_dpp(0, (int)f2u(x), 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, true));
}
template <> __device__ __forceinline__ float lane_xor<4>(float x) {
    return u2f((uint32_t)__builtin_amdgcn_ds_swizzle((int)f2u(x), 0x101F /* bit mode: and 0x1F, or 0, xor 4 */));
}

// One group-combining stage when the groups of a block sit in consecutive lanes (group j of the block in lane l with
// l % nb == j).  Both lanes of a pair form partner * t + own in one fused multiply-add, t = +1 in the lower lane (a + b),
// t = -1 in the upper lane (-(a - b)): multiplying by +-1 is exact and rounding is symmetric in sign, so the bits are those
// of a + b and a - b, and a lane's values carry the sign (-1)^(stages in which it was the upper one).  The partners of
// every stage have been upper equally often before it; the transforms that follow are linear; block_norm_signed() takes
// the sign back in the final normalization.  For partners inside a quad the lane exchange rides in the instruction
// (written out: the compiler keeps a separate lane move; a DPP operand must not be read in the two issue slots after a
// vector instruction wrote it, hence the s_nop in front of four independent ones).  Every lane of the wave must take part.
#define QUARTET_STAGE4_DPP(CTRL_TEXT, a, b, c, d, t)                                                  \
    asm volatile("s_nop 1\n\t"                                                                         \
                 "v_fmac_f32_dpp %0, %0, %4 " CTRL_TEXT " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"  \
                 "v_fmac_f32_dpp %1, %1, %4 " CTRL_TEXT " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"  \
                 "v_fmac_f32_dpp %2, %2, %4 " CTRL_TEXT " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"  \
                 "v_fmac_f32_dpp %3, %3, %4 " CTRL_TEXT " row_mask:0xf bank_mask:0xf bound_ctrl:1"       \
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "v"(t))
template <int XOR> __device__ __forceinline__ void cross_lane_stage(float (&v)[32], uint32_t lane) {
    const float t = (lane & (uint32_t)XOR) ? -1.0f : 1.0f;
    if (XOR == 4) {
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = __builtin_fmaf(lane_xor<4>(v[i]), t, v[i]);
    } else {
#pragma unroll
        for (int i = 0; i < 32; i += 4) {
            if (XOR == 1) QUARTET_STAGE4_DPP("quad_perm:[1,0,3,2]", v[i], v[i + 1], v[i + 2], v[i + 3], t);
            else QUARTET_STAGE4_DPP("quad_perm:[2,3,0,1]", v[i], v[i + 1], v[i + 2], v[i + 3], t);
        }
    }
}
__device__ __forceinline__ void cross_lane_stages(float (&v)[32], uint32_t lane, uint32_t nb) {
    if (nb > 1u) cross_lane_stage<1>(v, lane);
    if (nb > 2u) cross_lane_stage<2>(v, lane);
    if (nb > 4u) cross_lane_stage<4>(v, lane);
}
// fl(1/sqrt(32 nb)) with the sign the lane's values carry after cross_lane_stages.  Use it as
// fma(v, block_norm_signed, +0): the added +0 makes a zero of either sign +0, which is what the sums and differences of
// the unsigned values give.
__device__ __forceinline__ float block_norm_signed(uint32_t nb, uint32_t lane) {
    const uint32_t j = lane & (nb - 1u);
    return ((j ^ (j >> 1) ^ (j >> 2)) & 1u) ? -block_norm(nb) : block_norm(nb);
}

// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> four 32-bit words.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        // a ^ b ^ c in one three-input bit operation (truth table 0x96) instead of two XORs
        uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Stochastic rounding of eight values (|v| < 6) onto the E2M1 grid, packed into one dword, element j
// in bits [4j, 4j+4) (Section 3, "Rounding").  Rule: with lo <= |v| < hi adjacent grid points and
// f = (|v|-lo)/(hi-lo), the result is hi iff floor(f 2^22) + r >= 2^22 for the element's 22-bit draw r.
// Draws: a 32-bit Philox word serves four elements; element t owns byte t and rotates the word so that
// its byte leads: R = rotr(w, 8t + 8), r = R >> 10.  w0 serves elements 0..3, w1 elements 4..7.
// v_cvt_scalef32_sr_pk_fp4_f32 was measured on gfx950 to compute exactly
//     floor(f 2^22) + R[31:10] >= 2^22
// for the first value of its pair with R = its 32-bit random operand, and the same with R << 1 for
// the second value (all binades down to 2^-16, thresholds probed to +-1); the two values of a pair
// therefore share random bits, so each pair is converted twice, once with the even element's R and
// once with the odd element's R rotated right by one more bit (so that R << 1 shows its bits 31:10),
// and the valid nibbles are merged.
// One conversion of a pair into byte SEL of dst, keeping dst's other bytes.  Written as inline
// assembly because the destination must be tied to the previous partial result.
#define QUARTET_SR_CVT(SEL, OPSEL)                                                                 \
    template <> __device__ __forceinline__ void sr_cvt_pair<SEL>(uint32_t& dst, v2f pair, uint32_t rnd) { \
        asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:" OPSEL : "+v"(dst) : "v"(pair), "v"(rnd)); \
    }
template <int SEL> __device__ __forceinline__ void sr_cvt_pair(uint32_t& dst, v2f pair, uint32_t rnd);
QUARTET_SR_CVT(0, "[0,0,0,0]")
QUARTET_SR_CVT(1, "[0,0,1,0]")
QUARTET_SR_CVT(2, "[0,0,0,1]")
QUARTET_SR_CVT(3, "[0,0,1,1]")
#undef QUARTET_SR_CVT

__device__ __forceinline__ uint32_t rotr32(uint32_t x, uint32_t n) { return __builtin_amdgcn_alignbit(x, x, n); }

__device__ __forceinline__ uint32_t sr_pack8(const float* v, uint32_t w0, uint32_t w1) {
    uint32_t even, odd;      // every byte of both is written by a conversion below: no initial value needed
    asm volatile("" : "=v"(even));
    asm volatile("" : "=v"(odd));
    v2f p0 = {v[0], v[1]}, p1 = {v[2], v[3]}, p2 = {v[4], v[5]}, p3 = {v[6], v[7]};
    sr_cvt_pair<0>(even, p0, rotr32(w0, 8u));     // element 0: byte 0 leads
    sr_cvt_pair<1>(even, p1, rotr32(w0, 24u));    // element 2
    sr_cvt_pair<2>(even, p2, rotr32(w1, 8u));     // element 4
    sr_cvt_pair<3>(even, p3, rotr32(w1, 24u));    // element 6
    sr_cvt_pair<0>(odd, p0, rotr32(w0, 17u));     // element 1: rotr 16, one more for the instruction's R << 1
    sr_cvt_pair<1>(odd, p1, rotr32(w0, 1u));      // element 3: rotr 32 = 0, one more
    sr_cvt_pair<2>(odd, p2, rotr32(w1, 17u));     // element 5
    sr_cvt_pair<3>(odd, p3, rotr32(w1, 1u));      // element 7
    return (even & 0x0F0F0F0Fu) | (odd & 0xF0F0F0F0u);
}

}  // namespace quartet
