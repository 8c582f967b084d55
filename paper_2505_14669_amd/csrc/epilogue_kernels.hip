// Gradient epilogue of Algorithm 1 Backward: out = scale * H_32( g . M ) along the row,
// H_32 being its own inverse.  One lane owns one group of 32 fp32 values (128 bytes); a wave
// stages its 64 groups (8 KB) through LDS so that global loads are lane-contiguous.
#include "device_common.h"
#include "launchers.h"

namespace quartet {

__device__ __forceinline__ uint32_t pack_bf16x2_rne(float lo, float hi) {
    uint32_t a = f2u(lo), b = f2u(hi);
    a += 0x7FFFu + ((a >> 16) & 1u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xFFFF0000u);
}

// NB > 1: the Hadamard block spans nb = 2, 4 or 8 groups held by consecutive lanes (a row's groups start
// at a multiple of nb), combined across lanes before the 32-point stages.
template <bool OUT_BF16, bool MASK, bool BIG>
__global__ void __launch_bounds__(256)
grad_epilogue_kernel(const uint4* g, const uint32_t* __restrict__ mask, uint32_t n_groups,
                     float scale, void* out, uint32_t nb) {
    __shared__ uint4 stage[4][512];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    const uint32_t base_group = (blockIdx.x * 4u + wave) * 64u;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j) {
        uint32_t c = 64u * j + lane;                       // 16-byte chunk in the wave's 8 KB
        uint32_t grp = base_group + (c >> 3);
        uint4 q = (grp < n_groups) ? load_stream16(&g[(size_t)base_group * 8u + c]) : zero;
        stage[wave][(c & ~7u) | ((c & 7u) ^ ((c >> 4) & 7u))] = q;
    }
    __syncthreads();
    float v[32];
#pragma unroll
    for (uint32_t j = 0; j < 8; ++j) {
        uint4 q = stage[wave][8u * lane + (j ^ ((lane >> 1) & 7u))];
        v[4 * j] = u2f(q.x); v[4 * j + 1] = u2f(q.y); v[4 * j + 2] = u2f(q.z); v[4 * j + 3] = u2f(q.w);
    }
    const uint32_t grp = base_group + lane;
    if (MASK) {
        uint32_t mw = (grp < n_groups) ? mask[grp] : 0u;
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = ((mw >> i) & 1u) ? v[i] : 0.0f;
    }
    if (BIG) {
        cross_lane_stages(v, lane, nb);
        fwht32_unscaled(v);
        const float c = block_norm_signed(nb, lane);
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = __builtin_fmaf(v[i], c, 0.0f);
    } else {
        fwht32(v);
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = v[i] * scale;
    if (grp >= n_groups) return;
    if (OUT_BF16) {
        uint4* dst = reinterpret_cast<uint4*>(static_cast<uint16_t*>(out) + (size_t)grp * 32u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            dst[j] = make_uint4(pack_bf16x2_rne(v[8 * j], v[8 * j + 1]), pack_bf16x2_rne(v[8 * j + 2], v[8 * j + 3]),
                                pack_bf16x2_rne(v[8 * j + 4], v[8 * j + 5]), pack_bf16x2_rne(v[8 * j + 6], v[8 * j + 7]));
    } else {
        float4* dst = reinterpret_cast<float4*>(static_cast<float*>(out) + (size_t)grp * 32u);
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[j] = make_float4(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
    }
}

template <bool OUT_BF16, bool MASK>
static void launch_epilogue_nb(dim3 grid, hipStream_t st, const uint4* gp, const uint32_t* mask, uint32_t n_groups,
                               float scale, void* out, uint32_t nb) {
    dim3 block(256);
    if (nb > 1u) hipLaunchKernelGGL((grad_epilogue_kernel<OUT_BF16, MASK, true>), grid, block, 0, st, gp, mask, n_groups, scale, out, nb);
    else hipLaunchKernelGGL((grad_epilogue_kernel<OUT_BF16, MASK, false>), grid, block, 0, st, gp, mask, n_groups, scale, out, nb);
}

hipError_t launch_grad_epilogue(const float* g, const uint32_t* mask, int64_t m, int64_t n, uint32_t nb, float scale,
                                void* out, int out_bf16, hipStream_t st) {
    uint64_t n_groups = (uint64_t)m * (uint64_t)(n / 32);
    if (n_groups == 0) return hipSuccess;
    uint32_t tiles = (uint32_t)((n_groups + 63) / 64);
    dim3 grid((tiles + 3) / 4);
    const uint4* gp = reinterpret_cast<const uint4*>(g);
    if (out_bf16) {
        if (mask) launch_epilogue_nb<true, true>(grid, st, gp, mask, (uint32_t)n_groups, scale, out, nb);
        else launch_epilogue_nb<true, false>(grid, st, gp, mask, (uint32_t)n_groups, scale, out, nb);
    } else {
        if (mask) launch_epilogue_nb<false, true>(grid, st, gp, mask, (uint32_t)n_groups, scale, out, nb);
        else launch_epilogue_nb<false, false>(grid, st, gp, mask, (uint32_t)n_groups, scale, out, nb);
    }
    return hipGetLastError();
}

}  // namespace quartet
