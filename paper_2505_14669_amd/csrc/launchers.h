// Host-side launch functions of the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quartet {

// randomized-Hadamard sign words, Philox key/stream and Hadamard block of one quantizer call
struct SrParams {
    uint32_t sign_word;        // sign bits of a 32-element block (= sign_words[0])
    uint32_t key0, key1;
    uint32_t stream_id;
    uint32_t nb;               // groups per Hadamard block: 1 (the method's g = 32), 2, 4 or 8
    uint32_t sign_words[8];    // sign bits of a block of 32 nb elements, word j for its group j
};

hipError_t launch_quant(int mode, const void* x, int64_t rows, int64_t k, int64_t ldx, int transpose,
                        const SrParams& p, uint8_t* codes, uint8_t* scales, uint32_t* mask, hipStream_t st);
hipError_t launch_requant_transpose(int mode, const uint8_t* src_codes, const uint8_t* src_scales,
                                    int64_t rows, int64_t k, const SrParams& p, uint8_t* codes,
                                    uint8_t* scales, hipStream_t st);
// X [tokens x in] and W [out x in] quantized by the forward rule in one launch (Hadamard block 32, masks written)
hipError_t launch_fwd_operands(const void* x, int64_t tokens, const void* w, int64_t out, int64_t in, uint8_t* xq_codes,
                               uint8_t* xq_scales, uint32_t* x_mask, uint8_t* wq_codes, uint8_t* wq_scales, uint32_t* w_mask,
                               const SrParams& p, hipStream_t st);
// dy^T quantized along the tokens, X_q and W_q re-quantized along their other dimension: one launch (Hadamard block 32);
// with dy_codes != null also dy itself quantized along out (parameters p_dy) in the same launch
hipError_t launch_bwd_operands(int mode, const void* dy, int64_t tokens, int64_t in, int64_t out,
                               const uint8_t* xq_codes, const uint8_t* xq_scales, const uint8_t* wq_codes, const uint8_t* wq_scales,
                               const SrParams& p_dyt, const SrParams& p_x, const SrParams& p_w,
                               uint8_t* dyt_codes, uint8_t* dyt_scales, uint8_t* xt_codes, uint8_t* xt_scales,
                               uint8_t* wt_codes, uint8_t* wt_scales,
                               const SrParams& p_dy, uint8_t* dy_codes, uint8_t* dy_scales, hipStream_t st);
hipError_t launch_dequant(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t k, float* out,
                          hipStream_t st);
hipError_t launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                       const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                       int d_bf16, int64_t ldd, int fused, const uint32_t* mask, uint32_t nb, hipStream_t st);
// two gradient products (fused epilogue, same result type) in one launch where the tile-shape heuristic allows it
struct GemmArgs {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* b_codes;
    const uint8_t* b_scales;
    int64_t m, n, k;
    float alpha;
    void* d;
    int64_t ldd;
    const uint32_t* mask;
};
hipError_t launch_gemm_grad_pair(const GemmArgs& g0, const GemmArgs& g1, int d_bf16, uint32_t nb, hipStream_t st);
// variant: -1 = size heuristic, 0..2 = force that tile shape (256x256, 128x256, 128x128); band_height: 0 = heuristic, > 0 = tile rows per band
void set_gemm_plan(int variant, int band_height);
hipError_t launch_grad_epilogue(const float* g, const uint32_t* mask, int64_t m, int64_t n, uint32_t nb, float scale,
                                void* out, int out_bf16, hipStream_t st);

// measurement support: register-only loop of the FP4 matrix-core instruction (probe_kernels.hip); device counters
// {shader-clock ticks, constant-clock ticks} that the streaming GEMM kernel and the probe add their blocks' run time to
hipError_t launch_mfma_ceiling(const uint8_t* codes, const uint8_t* scales, uint32_t iterations, uint32_t blocks, float* sink,
                               uint64_t* counters, hipStream_t st);
void set_clock_counters(uint64_t* device_counters);

// MXFP8 comparison path (E4M3 elements, E8M0 scale per 32)
hipError_t launch_mxfp8_quant(const void* x, int64_t rows, int64_t k, int64_t ldx, uint8_t* codes, uint8_t* scales,
                              hipStream_t st);
hipError_t launch_mxfp8_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                             const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                             int d_bf16, int64_t ldd, hipStream_t st);

}  // namespace quartet
