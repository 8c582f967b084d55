// Measurement support (no step of the method): what the block-scaled FP4 matrix-core instruction sustains on this chip
// when nothing but the instruction runs -- operands in registers, no LDS, no memory traffic in the loop.  The GEMM's
// roofline fraction is reported next to this ceiling, measured in the same process on the same box.
#include "device_common.h"
#include "launchers.h"

namespace quartet {

// Shader-clock and constant-clock ticks a block spent between two points, added to counters[0] and counters[1]
// (the GEMM kernel records the same pair): their ratio times the constant clock's rate is the shader clock the
// chip held while the kernel ran.
__device__ __forceinline__ void clock_begin(const uint64_t* counters, uint64_t& t0, uint64_t& w0) {
    if (counters) {
        t0 = __builtin_readcyclecounter();
        w0 = __builtin_amdgcn_s_memrealtime();
    }
}
__device__ __forceinline__ void clock_end(uint64_t* counters, uint64_t t0, uint64_t w0) {
    if (counters && threadIdx.x == 0) {
        const uint64_t t1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
        atomicAdd(reinterpret_cast<unsigned long long*>(counters), (unsigned long long)(t1 - t0));
        atomicAdd(reinterpret_cast<unsigned long long*>(counters) + 1, (unsigned long long)(w1 - w0));
    }
}

// Each wave keeps the GEMM kernel's 4 x 4 accumulator tiles and issues `iterations` rounds of the 16
// v_mfma_scale_f32_32x32x64_f8f6f4 of one K-step on four A and four B fragments it loaded once (lane l of a block:
// fragment f is codes[(f*256 + l)*16 .. +16), scale dword scales[(f*256 + l)*4 .. +4)).
__global__ void __launch_bounds__(256)
mfma_ceiling_kernel(const uint4* __restrict__ codes, const uint32_t* __restrict__ scales, uint32_t iterations,
                    float* __restrict__ sink, uint64_t* __restrict__ counters) {
    uint64_t t0 = 0, w0 = 0;
    clock_begin(counters, t0, w0);
    uint4 fa[4], fb[4];
    uint32_t sa[4], sb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[i] = codes[i * 256 + threadIdx.x];
        fb[i] = codes[(4 + i) * 256 + threadIdx.x];
        sa[i] = scales[i * 256 + threadIdx.x];
        sb[i] = scales[(4 + i) * 256 + threadIdx.x];
    }
    v16f acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (uint32_t it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v8i a = {(int)fa[i].x, (int)fa[i].y, (int)fa[i].z, (int)fa[i].w, 0, 0, 0, 0};
                const v8i b = {(int)fb[j].x, (int)fb[j].y, (int)fb[j].z, (int)fb[j].w, 0, 0, 0, 0};
                acc[i * 4 + j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i * 4 + j], 4, 4, 0, (int)sa[i], 0, (int)sb[j]);
            }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    clock_end(counters, t0, w0);
}

hipError_t launch_mfma_ceiling(const uint8_t* codes, const uint8_t* scales, uint32_t iterations, uint32_t blocks, float* sink,
                               uint64_t* counters, hipStream_t st) {
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(blocks), dim3(256), 0, st, reinterpret_cast<const uint4*>(codes),
                       reinterpret_cast<const uint32_t*>(scales), iterations, sink, counters);
    return hipGetLastError();
}

}  // namespace quartet
