// MXFP4 x MXFP4 -> fp32 GEMM on the gfx950 block-scaled matrix cores (Section 4.4, "Stage 2":
// D = (A x SFA)(B x SFB)^T with one E8M0 scale per 32 elements along K).
//
// v_mfma_scale_f32_32x32x64_f8f6f4 operand layout (FP4, cbsz = blgp = 4), measured on gfx950:
//   A: lane l holds row l%32, K-elements 32*(l/32) .. +31 as 128 bits, element j in bits [4j,4j+4)
//      -- exactly the packed row-major code bytes, so a fragment is one 16-byte LDS read;
//   B: the same with the output column in place of the row;
//   scale: one byte per lane (selected by op_sel from a 32-bit register) = the E8M0 scale of that
//      lane's 32 K-elements, i.e. one MX group per lane per instruction;
//   D: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32.
// The tiled scale layout (see scale_tile_offset) stores, for each block of 32 rows and 256
// K-elements, one dword per lane whose four bytes are that lane's scales for the four K=64 steps,
// so a wave's scale fragment is one coalesced 256-byte global load and the paper's separate
// scale-rearrangement step does not exist here.
//
// Kernel shape: block tile BM x BN, K staged through LDS 256 elements (128 code bytes per row) at a
// time, two LDS buffers, global loads for stage t+1 issued before the matrix-core work of stage t.
#include "device_common.h"
#include "launchers.h"

#include <stdlib.h>

namespace quartet {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int S>
__device__ __forceinline__ v16f mfma_fp4(const uint4& a, const uint4& b, v16f c, uint32_t sa, uint32_t sb) {
    v8i va = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    v8i vb = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, c, 4, 4, S, (int)sa, S, (int)sb);
}

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Raw buffer resource over [base, base + bytes): loads past the end return zero, which is how ragged
// tile edges are handled without per-load predicates.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset no resource here reaches

template <int WAVES_M, int WAVES_N, int TM, int TN, bool OUT_BF16>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64)
gemm_mxfp4_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
                  const uint8_t* __restrict__ b_codes, const uint8_t* __restrict__ b_scales,
                  uint32_t m, uint32_t n, uint32_t k, float alpha, void* __restrict__ d, int64_t ldd,
                  uint32_t tiles_m, uint32_t tiles_n) {
    constexpr uint32_t NT = WAVES_M * WAVES_N * 64;
    constexpr uint32_t BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    constexpr uint32_t LA = BM * 8 / NT, LB = BN * 8 / NT;   // 16-byte chunks each thread moves per stage
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0 && (NT / 8) % 8 == 0, "tile/threads mismatch");
    __shared__ uint4 lds[2][(BM + BN) * 8];

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;

    // XCD-aware tile order: consecutive block ids land on different XCDs (8, round-robin), so give
    // each XCD one contiguous range of tiles, and walk tiles in bands of 8 tile-rows so that the
    // blocks running together on an XCD share A and B panels in its L2.
    uint32_t tile;
    {
        const uint32_t nb = gridDim.x, xcd = blockIdx.x & 7u, q = blockIdx.x >> 3;
        const uint32_t per = nb >> 3, rem = nb & 7u;
        tile = xcd * per + (xcd < rem ? xcd : rem) + q;
    }
    constexpr uint32_t GM = 8;
    const uint32_t band = tile / (GM * tiles_n);
    const uint32_t band_rows = (tiles_m - band * GM) < GM ? (tiles_m - band * GM) : GM;
    const uint32_t in_band = tile - band * GM * tiles_n;
    const uint32_t m0 = (band * GM + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;
    const uint32_t wm0 = (wave / WAVES_N) * (TM * 32), wn0 = (wave % WAVES_N) * (TN * 32);

    const uint32_t kb = k >> 1, gk = k >> 5, kq = (k + 255u) >> 8;   // code bytes, groups, K-quads per row
    const uint32_t rows_a = (m - m0) < BM ? (m - m0) : BM, rows_b = (n - n0) < BN ? (n - n0) : BN;

    const __amdgpu_buffer_rsrc_t res_a = make_rsrc(a_codes + (size_t)m0 * kb, rows_a * kb);
    const __amdgpu_buffer_rsrc_t res_b = make_rsrc(b_codes + (size_t)n0 * kb, rows_b * kb);
    // scale tiles: [row block][K-quad][lane][4 bytes]
    const __amdgpu_buffer_rsrc_t res_sa = make_rsrc(a_scales + (size_t)(m0 >> 5) * kq * 256u, ((rows_a + 31u) >> 5) * kq * 256u);
    const __amdgpu_buffer_rsrc_t res_sb = make_rsrc(b_scales + (size_t)(n0 >> 5) * kq * 256u, ((rows_b + 31u) >> 5) * kq * 256u);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // this thread's chunk: row tid/8 (+ j*NT/8), 16-byte column tid%8 of the 128-byte stage row
    const uint32_t crow = tid >> 3, ccol = tid & 7u;
    const uint32_t goff = crow * kb + ccol * 16u;               // byte offset inside the tile's rows
    const uint32_t gstep = (NT / 8u) * kb;                       // + j * gstep for the j-th chunk
    const uint32_t lpos = crow * 8u + (ccol ^ (crow & 7u));     // LDS chunk position (+ j * NT)
    const uint32_t soff_a = ((wm0 >> 5) * kq * 64u + lane) * 4u;  // + i * kq*256 per 32-row block, + st*256
    const uint32_t soff_b = ((wn0 >> 5) * kq * 64u + lane) * 4u;
    const uint32_t sstep = kq * 256u;

    const uint32_t stages = kq;
    v4u ra[LA], rb[LB];
    uint32_t sa[TM], sb[TN], sa_n[TM], sb_n[TN];

#define QUARTET_LOAD_STAGE(ST, XA, XB)                                                                  \
    {                                                                                                   \
        const uint32_t st_ = (ST);                                                                      \
        const uint32_t base_ = (st_ * 128u + ccol * 16u < kb) ? goff + st_ * 128u : kOutOfRange;        \
        _Pragma("unroll") for (uint32_t j = 0; j < LA; ++j)                                             \
            ra[j] = __builtin_amdgcn_raw_buffer_load_b128(res_a, base_ + j * gstep, 0, 0);              \
        _Pragma("unroll") for (uint32_t j = 0; j < LB; ++j)                                             \
            rb[j] = __builtin_amdgcn_raw_buffer_load_b128(res_b, base_ + j * gstep, 0, 0);              \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i)                                             \
            XA[i] = __builtin_amdgcn_raw_buffer_load_b32(res_sa, soff_a + i * sstep + st_ * 256u, 0, 0); \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j)                                             \
            XB[j] = __builtin_amdgcn_raw_buffer_load_b32(res_sb, soff_b + j * sstep + st_ * 256u, 0, 0); \
        if (st_ == stages - 1u && (gk & 7u) != 0u) {                                                    \
            /* ragged K: groups past k/32 hold zero codes; neutralize whatever their scale bytes hold */ \
            uint32_t keep = 0u;                                                                         \
            _Pragma("unroll") for (uint32_t p = 0; p < 4; ++p)                                          \
                if (st_ * 8u + 2u * p + lhalf < gk) keep |= 0xFFu << (8u * p);                          \
            _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) XA[i] = (XA[i] & keep) | (0x7F7F7F7Fu & ~keep); \
            _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) XB[j] = (XB[j] & keep) | (0x7F7F7F7Fu & ~keep); \
        }                                                                                               \
    }
#define QUARTET_STORE_STAGE(BUF)                                                                        \
    {                                                                                                   \
        _Pragma("unroll") for (uint32_t j = 0; j < LA; ++j)                                             \
            lds[BUF][lpos + j * NT] = make_uint4(ra[j].x, ra[j].y, ra[j].z, ra[j].w);                   \
        _Pragma("unroll") for (uint32_t j = 0; j < LB; ++j)                                             \
            lds[BUF][BM * 8u + lpos + j * NT] = make_uint4(rb[j].x, rb[j].y, rb[j].z, rb[j].w);         \
    }
#define QUARTET_KSTEP(S)                                                                                \
    {                                                                                                   \
        uint4 fa[TM], fb[TN];                                                                           \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) {                                           \
            uint32_t row = wm0 + i * 32u + lrow;                                                        \
            fa[i] = sA[row * 8u + ((2u * S + lhalf) ^ (row & 7u))];                                     \
        }                                                                                               \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) {                                           \
            uint32_t row = wn0 + j * 32u + lrow;                                                        \
            fb[j] = sB[row * 8u + ((2u * S + lhalf) ^ (row & 7u))];                                     \
        }                                                                                               \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i)                                             \
            _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j)                                         \
                acc[i][j] = mfma_fp4<S>(fa[i], fb[j], acc[i][j], sa[i], sb[j]);                         \
        if (NT > 256) __builtin_amdgcn_sched_barrier(0); /* two waves per SIMD: keep fragments of one K-step live at a time */ \
    }

    if (stages > 0) {
        QUARTET_LOAD_STAGE(0u, sa, sb)
        QUARTET_STORE_STAGE(0)
    }
    __syncthreads();

    for (uint32_t st = 0; st < stages; ++st) {
        const uint32_t buf = st & 1u;
        const bool more = st + 1u < stages;
        if (more) QUARTET_LOAD_STAGE(st + 1u, sa_n, sb_n)
        const uint4* sA = &lds[buf][0];
        const uint4* sB = &lds[buf][BM * 8];
        QUARTET_KSTEP(0)
        QUARTET_KSTEP(1)
        QUARTET_KSTEP(2)
        QUARTET_KSTEP(3)
        if (more) {
            QUARTET_STORE_STAGE(buf ^ 1u)
#pragma unroll
            for (uint32_t i = 0; i < TM; ++i) sa[i] = sa_n[i];
#pragma unroll
            for (uint32_t j = 0; j < TN; ++j) sb[j] = sb_n[j];
        }
        __syncthreads();
    }
#undef QUARTET_LOAD_STAGE
#undef QUARTET_STORE_STAGE
#undef QUARTET_KSTEP

#pragma unroll
    for (uint32_t i = 0; i < TM; ++i)
#pragma unroll
        for (uint32_t j = 0; j < TN; ++j) {
            uint32_t col = n0 + wn0 + j * 32u + lrow;
#pragma unroll
            for (uint32_t r = 0; r < 16; ++r) {
                uint32_t row = m0 + wm0 + i * 32u + (r >> 2) * 8u + lhalf * 4u + (r & 3u);
                if (row < m && col < n) {
                    float val = alpha * acc[i][j][r];
                    if (OUT_BF16)
                        static_cast<uint16_t*>(d)[(size_t)row * ldd + col] = f32_to_bf16_rne(val);
                    else
                        static_cast<float*>(d)[(size_t)row * ldd + col] = val;
                }
            }
        }
}

template <int WAVES_M, int WAVES_N, int TM, int TN>
static hipError_t launch_variant(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                                 const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha,
                                 void* d, int d_bf16, int64_t ldd, hipStream_t st) {
    constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
    uint32_t tiles_m = (uint32_t)((m + BM - 1) / BM), tiles_n = (uint32_t)((n + BN - 1) / BN);
    dim3 grid(tiles_m * tiles_n), block(WAVES_M * WAVES_N * 64);
    const uint8_t *as = a_scales, *bs = b_scales;
    if (d_bf16)
        hipLaunchKernelGGL((gemm_mxfp4_kernel<WAVES_M, WAVES_N, TM, TN, true>), grid, block, 0, st, a_codes, as,
                           b_codes, bs, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, ldd, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((gemm_mxfp4_kernel<WAVES_M, WAVES_N, TM, TN, false>), grid, block, 0, st, a_codes, as,
                           b_codes, bs, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, ldd, tiles_m, tiles_n);
    return hipGetLastError();
}

// Tile shapes: 0 = 256x256 (8 waves, 128x64 each), 1 = 256x256 (4 waves, 128x128 each),
// 2 = 128x128 (4 waves, 64x64 each).  QUARTET_GEMM_VARIANT overrides the size heuristic (tuning aid).
hipError_t launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                       const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                       int d_bf16, int64_t ldd, hipStream_t st) {
    if (m == 0 || n == 0) return hipSuccess;
    const char* env = getenv("QUARTET_GEMM_VARIANT");
    int variant = (env && *env) ? atoi(env) : -1;
    if (variant < 0) {
        int64_t big_tiles = ((m + 255) / 256) * ((n + 255) / 256);
        variant = big_tiles >= 192 ? 0 : 2;
    }
    switch (variant) {
    case 0: return launch_variant<2, 4, 4, 2>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, d_bf16, ldd, st);
    case 1: return launch_variant<2, 2, 4, 4>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, d_bf16, ldd, st);
    default: return launch_variant<2, 2, 2, 2>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, d_bf16, ldd, st);
    }
}

}  // namespace quartet
