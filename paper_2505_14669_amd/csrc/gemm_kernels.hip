// MXFP4 x MXFP4 -> fp32 GEMM on the gfx950 block-scaled matrix cores (Section 4.4, "Stage 2":
// D = (A x SFA)(B x SFB)^T with one E8M0 scale per 32 elements along K).
//
// v_mfma_scale_f32_32x32x64_f8f6f4 operand layout (FP4, cbsz = blgp = 4), measured on gfx950:
//   A: lane l holds row l%32, K-elements 32*(l/32) .. +31 as 128 bits, element j in bits [4j,4j+4)
//      -- exactly the packed row-major code bytes, so a fragment is one 16-byte LDS read;
//   B: the same with the output column in place of the row;
//   scale: one byte per lane (selected by opsel from a 32-bit register) = the E8M0 scale of that
//      lane's 32 K-elements, i.e. one MX group per lane per instruction;
//   D: lane l, register r -> row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "device_common.h"
#include "launchers.h"

namespace quartet {

constexpr int kBK = 128;             // K elements per LDS stage = 64 code bytes = 4 chunks of 16 B

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool OUT_BF16>
__global__ void __launch_bounds__(WAVES_M * WAVES_N * 64)
gemm_mxfp4_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
                  const uint8_t* __restrict__ b_codes, const uint8_t* __restrict__ b_scales,
                  uint32_t m, uint32_t n, uint32_t k, float alpha, void* __restrict__ d, int64_t ldd) {
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    __shared__ uint4 sA[BM * 4];
    __shared__ uint4 sB[BN * 4];

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
    const uint32_t m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const uint32_t kb = k >> 1, gk = k >> 5;             // code bytes / scale bytes per row
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const uint32_t k_tiles = (k + kBK - 1) / kBK;
    for (uint32_t kt = 0; kt < k_tiles; ++kt) {
        // global -> LDS, 16-byte chunks, swizzled so that fragment reads are conflict-free
#pragma unroll
        for (int id0 = 0; id0 < BM * 4; id0 += NT) {
            uint32_t id = id0 + tid;
            if (BM * 4 % NT == 0 || id < BM * 4) {
                uint32_t row = id >> 2, c = id & 3u;
                uint32_t grow = m0 + row, kbyte = kt * 64u + c * 16u;
                uint4 q = zero4;
                if (grow < m && kbyte < kb)
                    q = *reinterpret_cast<const uint4*>(a_codes + (size_t)grow * kb + kbyte);
                sA[row * 4u + (c ^ ((row >> 1) & 3u))] = q;
            }
        }
#pragma unroll
        for (int id0 = 0; id0 < BN * 4; id0 += NT) {
            uint32_t id = id0 + tid;
            if (BN * 4 % NT == 0 || id < BN * 4) {
                uint32_t row = id >> 2, c = id & 3u;
                uint32_t grow = n0 + row, kbyte = kt * 64u + c * 16u;
                uint4 q = zero4;
                if (grow < n && kbyte < kb)
                    q = *reinterpret_cast<const uint4*>(b_codes + (size_t)grow * kb + kbyte);
                sB[row * 4u + (c ^ ((row >> 1) & 3u))] = q;
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t ks = 0; ks < 2; ++ks) {
            const uint32_t kblock = kt * 4u + ks * 2u + lhalf;  // this lane's MX group along K
            const bool kok = kblock < gk;
            v8i fa[TM], fb[TN];
            uint32_t sa[TM], sb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                uint32_t row = wm0 + i * 32u + lrow;
                uint4 q = sA[row * 4u + ((ks * 2u + lhalf) ^ ((row >> 1) & 3u))];
                fa[i] = (v8i){(int)q.x, (int)q.y, (int)q.z, (int)q.w, 0, 0, 0, 0};
                uint32_t grow = m0 + row;
                sa[i] = (kok && grow < m) ? (uint32_t)a_scales[(size_t)grow * gk + kblock] : 127u;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                uint32_t row = wn0 + j * 32u + lrow;
                uint4 q = sB[row * 4u + ((ks * 2u + lhalf) ^ ((row >> 1) & 3u))];
                fb[j] = (v8i){(int)q.x, (int)q.y, (int)q.z, (int)q.w, 0, 0, 0, 0};
                uint32_t grow = n0 + row;
                sb[j] = (kok && grow < n) ? (uint32_t)b_scales[(size_t)grow * gk + kblock] : 127u;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[i], fb[j], acc[i][j], 4, 4, 0, (int)sa[i], 0, (int)sb[j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            uint32_t col = n0 + wn0 + j * 32u + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
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

hipError_t launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                       const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                       int d_bf16, int64_t ldd, hipStream_t st) {
    if (m == 0 || n == 0) return hipSuccess;
    constexpr int BM = 128, BN = 128;
    dim3 grid((uint32_t)((n + BN - 1) / BN), (uint32_t)((m + BM - 1) / BM)), block(256);
    if (d_bf16)
        hipLaunchKernelGGL((gemm_mxfp4_kernel<BM, BN, 2, 2, true>), grid, block, 0, st, a_codes, a_scales,
                           b_codes, b_scales, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, ldd);
    else
        hipLaunchKernelGGL((gemm_mxfp4_kernel<BM, BN, 2, 2, false>), grid, block, 0, st, a_codes, a_scales,
                           b_codes, b_scales, (uint32_t)m, (uint32_t)n, (uint32_t)k, alpha, d, ldd);
    return hipGetLastError();
}

}  // namespace quartet
