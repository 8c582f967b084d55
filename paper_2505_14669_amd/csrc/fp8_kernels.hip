// MXFP8 twin of the MXFP4 path, for the comparison the paper makes (Section 5, "Speedup results":
// MXFP4 linear layers against MXFP8 ones): E4M3 elements with one E8M0 scale per 32 along K
// (Section 3 names the format), plain absolute-maximum scaling, no rotation.  Same tiled scale
// layout, same 256 x 256 ring GEMM skeleton as the MXFP4 kernels; the matrix-core instruction is the
// same v_mfma_scale_f32_32x32x64_f8f6f4 with both operand formats set to FP8 (cbsz = blgp = 0), which
// runs at half the FP4 rate.
//
// FP8 operand layout of that instruction, measured on gfx950: lane l supplies row l%32 and 32 bytes;
// its first 16 bytes (registers 0-3) belong to K-elements 0..31 of the instruction, its last 16
// (registers 4-7) to K-elements 32..63, and inside each of the two 32-element blocks lanes 0..31 and
// lanes 32..63 hold one half each.  For a row stored as 64 contiguous bytes lane (row, h) therefore
// takes 16-byte chunks h and 2+h.  The scale byte of lane l applies to block l/32, as with FP4.
#include "gemm_common.h"
#include "launchers.h"

namespace quartet {

typedef short v2s_t __attribute__((ext_vector_type(2)));

// four values -> four E4M3 bytes, round-to-nearest-even; magnitudes above 448 saturate (the
// conversion itself would give NaN there)
__device__ __forceinline__ uint32_t e4m3_pack4(float a, float b, float c, float d) {
    a = __builtin_amdgcn_fmed3f(a, -448.0f, 448.0f);
    b = __builtin_amdgcn_fmed3f(b, -448.0f, 448.0f);
    c = __builtin_amdgcn_fmed3f(c, -448.0f, 448.0f);
    d = __builtin_amdgcn_fmed3f(d, -448.0f, 448.0f);
    v2s_t w = {0, 0};
    w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, a, b, 1.0f, false);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(w, c, d, 1.0f, true);
    return (uint32_t)(uint16_t)w[0] | ((uint32_t)(uint16_t)w[1] << 16);
}

// ------------------------------------------------------------------ quantizer, row mode
// Same block shape as the MXFP4 row quantizer: 8 rows x 32 groups, one lane per group, loads
// swizzled through LDS, scale bytes exchanged through LDS into whole runs of the scale tiles.
__global__ void __launch_bounds__(256)
mxfp8_quant_kernel(const uint16_t* __restrict__ x, uint32_t rows, uint32_t gk, int64_t ldx,
                   uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint32_t k_blocks, FastDiv div_k_blocks) {
    __shared__ uint4 stage[4][256];
    __shared__ uint32_t s_scale[64];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t row_set = fast_div(blockIdx.x, div_k_blocks);
    const uint32_t row0 = row_set * 8u, kq0 = (blockIdx.x - row_set * k_blocks) * 4u, kqs = (gk + 7u) >> 3;
    const uint32_t rows_here = (rows - row0) < 8u ? (rows - row0) : 8u;
    const __amdgpu_buffer_rsrc_t res_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(x + (size_t)row0 * ldx), 0, (int)(((rows_here - 1u) * (uint32_t)ldx + gk * 32u) * 2u), 0x00020000);
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        uint32_t c = 64u * j + lane;
        const uint32_t voff = ((wave * 2u + (c >> 7)) * (uint32_t)ldx + kq0 * 256u + (c & 127u) * 8u) * 2u;
        v4u_t q = __builtin_amdgcn_raw_buffer_load_b128(res_x, (int)voff, 0, 2 /* non-temporal */);
        stage[wave][(c & ~3u) | ((c & 3u) ^ ((c >> 4) & 3u))] = make_uint4(q.x, q.y, q.z, q.w);
    }
    __syncthreads();
    float v[32];
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        const uint4 q = stage[wave][4u * lane + (j ^ ((lane >> 2) & 3u))];
        v[8 * j] = u2f(q.x << 16); v[8 * j + 1] = u2f(q.x & 0xFFFF0000u);
        v[8 * j + 2] = u2f(q.y << 16); v[8 * j + 3] = u2f(q.y & 0xFFFF0000u);
        v[8 * j + 4] = u2f(q.z << 16); v[8 * j + 5] = u2f(q.z & 0xFFFF0000u);
        v[8 * j + 6] = u2f(q.w << 16); v[8 * j + 7] = u2f(q.w & 0xFFFF0000u);
    }
    const uint32_t row_local = wave * 2u + (lane >> 5), gi = lane & 31u;
    const uint32_t row = row0 + row_local, g = kq0 * 8u + gi;
    // scale: the largest magnitude goes to the top binade [2^8, 2^9) of the element format
    float mx = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) mx = __builtin_fmaxf(mx, __builtin_fabsf(v[i]));
    const uint32_t E = (f2u(mx) >> 23) & 0xFFu;
    const uint32_t b = E >= 8u ? E - 8u : 0u;
    const float mult = u2f((254u - b) << 23);               // 2^(127-b), exact
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = e4m3_pack4(v[4 * i] * mult, v[4 * i + 1] * mult, v[4 * i + 2] * mult, v[4 * i + 3] * mult);
    reinterpret_cast<uint8_t*>(s_scale)[(((gi >> 3) * 2u + (gi & 1u)) * 8u + row_local) * 4u + ((gi & 7u) >> 1)] = (uint8_t)b;
    if (row < rows && g < gk) {
        uint8_t* dst = codes + ((size_t)row * gk + g) * 32u;
        store_stream16(dst, make_uint4(c[0], c[1], c[2], c[3]));
        store_stream16(dst + 16, make_uint4(c[4], c[5], c[6], c[7]));
    }
    __syncthreads();
    if (threadIdx.x < 64u) {
        const uint32_t t = threadIdx.x, kql = t >> 4, h = (t >> 3) & 1u, rl = t & 7u;
        const uint32_t r = row0 + rl, kq = kq0 + kql;
        if (r < rows && kq * 8u + h < gk) {
            uint8_t* dst = scales + scale_tile_offset(r, kq * 8u + h, kqs);
            const uint32_t w = s_scale[t];
            if (kq * 8u + 8u <= gk) {
                *reinterpret_cast<uint32_t*>(dst) = w;
            } else {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q)
                    if (kq * 8u + 2u * q + h < gk) dst[q] = (uint8_t)(w >> (8u * q));
            }
        }
    }
}

// ------------------------------------------------------------------ GEMM
__device__ __forceinline__ v16f mfma_fp8(const uint4& a_lo, const uint4& a_hi, const uint4& b_lo, const uint4& b_hi,
                                         v16f c, uint32_t sa, uint32_t sb) {
    v8i va = {(int)a_lo.x, (int)a_lo.y, (int)a_lo.z, (int)a_lo.w, (int)a_hi.x, (int)a_hi.y, (int)a_hi.z, (int)a_hi.w};
    v8i vb = {(int)b_lo.x, (int)b_lo.y, (int)b_lo.z, (int)b_lo.w, (int)b_hi.x, (int)b_hi.y, (int)b_hi.z, (int)b_hi.w};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, c, 0, 0, 0, (int)sa, 0, (int)sb);
}

// 256 x 256 block tile, 128 x 128 wave tile, ring of kRing LDS stages filled kRing-1 ahead, as the
// MXFP4 ring kernel; a stage is 64 K-elements = 64 code bytes per row, i.e. ONE matrix-core K-step
// (16 instructions per wave), so the two fragment sets alternate from stage to stage: the second
// half of a stage's instructions runs over the LDS reads of the next stage's fragments.
template <bool OUT_BF16>
__global__ void __launch_bounds__(256)
gemm_mxfp8_ring_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
                       const uint8_t* __restrict__ b_codes, const uint8_t* __restrict__ b_scales,
                       uint32_t m, uint32_t n, uint32_t k, float alpha, void* __restrict__ d, uint32_t ldd,
                       uint32_t tiles_m, uint32_t tiles_n) {
    constexpr uint32_t TM = 4, TN = 4, BM = 256, BN = 256;
    constexpr uint32_t CODES = (BM + BN) * 4;            // 16-byte chunks of codes per stage
    constexpr uint32_t STAGE = CODES + 256;              // + 16 scale tiles of 256 B
    constexpr uint32_t D = kRing - 1;
    constexpr uint32_t LOADS = 9;
    constexpr uint32_t KEEP = (D - 1) * LOADS;
    constexpr uint32_t WAIT_STAGE = 0x0F70u | (KEEP & 15u) | ((KEEP >> 4) << 14);
    __shared__ uint4 lds[kRing * STAGE];
    static_assert(kRing * STAGE * 16 >= 4 * TM * 32 * kEpiStride * 4, "the epilogue's per-wave scratch must fit in the ring");

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;

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
    const uint32_t wm0 = (wave >> 1) * 128u, wn0 = (wave & 1u) * 128u;

    const uint32_t kb = k, gk = k >> 5, kq = (k + 255u) >> 8;   // code bytes per row, groups, K-quads
    const uint32_t rows_a = (m - m0) < BM ? (m - m0) : BM, rows_b = (n - n0) < BN ? (n - n0) : BN;
    const v4i_t res_a = make_rsrc_words(a_codes + (size_t)m0 * kb, rows_a * kb);
    const v4i_t res_b = make_rsrc_words(b_codes + (size_t)n0 * kb, rows_b * kb);
    const bool scales_of_a = wave < 2u;
    const uint32_t srow0 = scales_of_a ? m0 : n0, srows = scales_of_a ? rows_a : rows_b;
    const v4i_t res_s = make_rsrc_words((scales_of_a ? a_scales : b_scales) + (size_t)(srow0 >> 5) * kq * 256u,
                                        ((srows + 31u) >> 5) * kq * 256u);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // same LDS image as the MXFP4 ring kernel: rows of 64 bytes, chunk c of row r at r*4 + (c ^ (r/4)%4)
    const uint32_t drow = wave * 16u + (lane >> 2);
    const uint32_t dcol = (lane & 3u) ^ ((drow >> 2) & 3u);
    const uint32_t goff = drow * kb + dcol * 16u;          // + j*64*kb, + stage*64
    const uint32_t gstep = 64u * kb;
    const uint32_t soff = (((wave & 1u) * 4u + (lane >> 4)) * kq) * 256u + (lane & 15u) * 16u;   // + quad*256
    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)&lds[0];
    const uint32_t swz = (lrow >> 2) & 3u;
    const uint32_t fa_base = (wm0 + lrow) * 4u, fb_base = BM * 4u + (wn0 + lrow) * 4u;
    const uint32_t sa_base = CODES * 4u + (wm0 >> 5) * 64u + lane;
    const uint32_t sb_base = CODES * 4u + 8u * 64u + (wn0 >> 5) * 64u + lane;

    const uint32_t stages = (k + 63u) >> 6;
    uint32_t sa[TM], sb[TN], sa_n[TM], sb_n[TN];
    uint4 fa0[TM][2], fb0[TN][2], fa1[TM][2], fb1[TN][2];

#define F8_ISSUE(ST, J)                                                                                 \
    {                                                                                                   \
        const uint32_t st_ = (ST);                                                                      \
        const uint32_t slot_ = lds0 + ((st_ % kRing) * STAGE + wave * 64u) * 16u;                       \
        if ((J) < 8u) {                                                                                 \
            const uint32_t base_ = (st_ * 64u + dcol * 16u < kb) ? goff + st_ * 64u : kOutOfRange;      \
            lds_direct_load16((J) < 4u ? res_a : res_b, base_ + ((J) & 3u) * gstep, slot_ + (J) * 4096u); \
        } else {                                                                                        \
            lds_direct_load16(res_s, (st_ < stages) ? soff + (st_ >> 2) * 256u : kOutOfRange, slot_ + CODES * 16u); \
        }                                                                                               \
    }
// fragment of row block I: chunks lhalf (K-elements 0..31 of the stage) and 2 + lhalf (32..63)
#define F8_FRAG_A(ST, FA, I)                                                                            \
    FA[I][0] = lds[((ST) % kRing) * STAGE + fa_base + (I) * 128u + (lhalf ^ swz)];                      \
    FA[I][1] = lds[((ST) % kRing) * STAGE + fa_base + (I) * 128u + ((2u + lhalf) ^ swz)];
#define F8_FRAG_B(ST, FB, J)                                                                            \
    FB[J][0] = lds[((ST) % kRing) * STAGE + fb_base + (J) * 128u + (lhalf ^ swz)];                      \
    FB[J][1] = lds[((ST) % kRing) * STAGE + fb_base + (J) * 128u + ((2u + lhalf) ^ swz)];
// the stage's scale byte of each row block (byte ST%4 of the K-quad's dword), 1.0 for groups past k/32
#define F8_READ_SCALES(ST, XA, XB)                                                                      \
    {                                                                                                   \
        const uint32_t st_ = (ST);                                                                      \
        const uint32_t* sbuf_ = reinterpret_cast<const uint32_t*>(&lds[(st_ % kRing) * STAGE]);         \
        const uint32_t sh_ = (st_ & 3u) * 8u;                                                           \
        const bool keep_ = st_ * 2u + lhalf < gk;                                                       \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i)                                             \
            XA[i] = keep_ ? ((sbuf_[sa_base + i * 64u] >> sh_) & 0xFFu) : 0x7Fu;                        \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j)                                             \
            XB[j] = keep_ ? ((sbuf_[sb_base + j * 64u] >> sh_) & 0xFFu) : 0x7Fu;                        \
    }
#define F8_MFMA_ROW(FA, FB, I)                                                                          \
    _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j)                                                 \
        acc[I][j] = mfma_fp8(FA[I][0], FA[I][1], FB[j][0], FB[j][1], acc[I][j], sa[I], sb[j]);
#define F8_PIN_ROW(I)                                                                                   \
    _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[I][j]));
#define F8_FENCE() __builtin_amdgcn_sched_barrier(0);
// One stage on fragment set (FA, FB); the next stage's fragments go to (FAN, FBN).
#define F8_STAGE(ST, FA, FB, FAN, FBN)                                                                  \
    F8_FENCE()                                                                                          \
    F8_ISSUE((ST) + D, 0u) F8_ISSUE((ST) + D, 1u) F8_ISSUE((ST) + D, 2u) F8_ISSUE((ST) + D, 3u) F8_ISSUE((ST) + D, 4u) \
    F8_FENCE()                                                                                          \
    F8_MFMA_ROW(FA, FB, 0)                                                                              \
    F8_PIN_ROW(0)                                                                                       \
    F8_FENCE()                                                                                          \
    F8_ISSUE((ST) + D, 5u) F8_ISSUE((ST) + D, 6u) F8_ISSUE((ST) + D, 7u) F8_ISSUE((ST) + D, 8u)         \
    F8_FENCE()                                                                                          \
    F8_MFMA_ROW(FA, FB, 1)                                                                              \
    F8_PIN_ROW(1)                                                                                       \
    F8_FENCE()                                                                                          \
    __builtin_amdgcn_s_waitcnt(WAIT_STAGE);                                                             \
    __builtin_amdgcn_s_barrier();                                                                       \
    F8_FENCE()                                                                                          \
    _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) { F8_FRAG_A((ST) + 1u, FAN, i) F8_FRAG_B((ST) + 1u, FBN, i) } \
    F8_READ_SCALES((ST) + 1u, sa_n, sb_n)                                                               \
    F8_MFMA_ROW(FA, FB, 2)                                                                              \
    F8_MFMA_ROW(FA, FB, 3)                                                                              \
    _Pragma("unroll") for (uint32_t g_ = 0; g_ < 8; ++g_) {                                             \
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
    }                                                                                                   \
    F8_PIN_ROW(2)                                                                                       \
    F8_PIN_ROW(3)                                                                                       \
    F8_FENCE()                                                                                          \
    _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) sa[i] = sa_n[i];                                \
    _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) sb[j] = sb_n[j];

#pragma unroll
    for (uint32_t s0 = 0; s0 < D; ++s0) {
#pragma unroll
        for (uint32_t j = 0; j < LOADS; ++j) F8_ISSUE(s0, j)
    }
    __builtin_amdgcn_s_waitcnt(WAIT_STAGE);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (uint32_t i = 0; i < TM; ++i) { F8_FRAG_A(0u, fa0, i) F8_FRAG_B(0u, fb0, i) }
    F8_READ_SCALES(0u, sa, sb)

    for (uint32_t st = 0; st < stages; st += 2u) {
        F8_STAGE(st, fa0, fb0, fa1, fb1)
        F8_STAGE(st + 1u, fa1, fb1, fa0, fb0)      // past the end of K when `stages` is odd: zero codes, scale 1
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the zero-filled stages issued past the end
#undef F8_ISSUE
#undef F8_FRAG_A
#undef F8_FRAG_B
#undef F8_READ_SCALES
#undef F8_MFMA_ROW
#undef F8_PIN_ROW
#undef F8_FENCE
#undef F8_STAGE

    __builtin_amdgcn_s_barrier();
    store_tile<TM, TN, OUT_BF16>(acc, reinterpret_cast<float*>(lds) + wave * (TM * 32u * kEpiStride), d, ldd, alpha,
                                 m0 + wm0, n0 + wn0, m, n, lane);
}

// ------------------------------------------------------------------ host-side launchers
static FastDiv fast_div_of(uint32_t d) {
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    uint64_t mul = ((((uint64_t)1 << l) - d) << 32) / d + 1;
    return FastDiv{(uint32_t)mul, l};
}

hipError_t launch_mxfp8_quant(const void* x, int64_t rows, int64_t k, int64_t ldx, uint8_t* codes, uint8_t* scales,
                              hipStream_t st) {
    if (rows == 0 || k == 0) return hipSuccess;
    const uint32_t gk = (uint32_t)(k / 32), k_blocks = (gk + 31) / 32;
    hipLaunchKernelGGL(mxfp8_quant_kernel, dim3((uint32_t)((rows + 7) / 8) * k_blocks), dim3(256), 0, st,
                       (const uint16_t*)x, (uint32_t)rows, gk, ldx, codes, scales, k_blocks, fast_div_of(k_blocks));
    return hipGetLastError();
}

hipError_t launch_mxfp8_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                             const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                             int d_bf16, int64_t ldd, hipStream_t st) {
    if (m == 0 || n == 0) return hipSuccess;
    const uint32_t tiles_m = (uint32_t)((m + 255) / 256), tiles_n = (uint32_t)((n + 255) / 256);
    if (d_bf16)
        hipLaunchKernelGGL((gemm_mxfp8_ring_kernel<true>), dim3(tiles_m * tiles_n), dim3(256), 0, st, a_codes, a_scales,
                           b_codes, b_scales, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, (uint32_t)ldd, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((gemm_mxfp8_ring_kernel<false>), dim3(tiles_m * tiles_n), dim3(256), 0, st, a_codes, a_scales,
                           b_codes, b_scales, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, (uint32_t)ldd, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace quartet
