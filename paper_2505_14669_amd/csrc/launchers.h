// Host-side launch functions of the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quartet {

// randomized-Hadamard sign word and Philox key/stream of one quantizer call
struct SrParams {
    uint32_t sign_word;
    uint32_t key0, key1;
    uint32_t stream_id;
};

hipError_t launch_quant(int mode, const void* x, int64_t rows, int64_t k, int64_t ldx, int transpose,
                        const SrParams& p, uint8_t* codes, uint8_t* scales, uint32_t* mask, hipStream_t st);
hipError_t launch_requant_transpose(int mode, const uint8_t* src_codes, const uint8_t* src_scales,
                                    int64_t rows, int64_t k, const SrParams& p, uint8_t* codes,
                                    uint8_t* scales, hipStream_t st);
hipError_t launch_dequant(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t k, float* out,
                          hipStream_t st);
hipError_t launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                       const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                       int d_bf16, int64_t ldd, int fused, const uint32_t* mask, hipStream_t st);
hipError_t launch_grad_epilogue(const float* g, const uint32_t* mask, int64_t m, int64_t n, float scale,
                                void* out, int out_bf16, hipStream_t st);

// MXFP8 comparison path (E4M3 elements, E8M0 scale per 32)
hipError_t launch_mxfp8_quant(const void* x, int64_t rows, int64_t k, int64_t ldx, uint8_t* codes, uint8_t* scales,
                              hipStream_t st);
hipError_t launch_mxfp8_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                             const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                             int d_bf16, int64_t ldd, hipStream_t st);

}  // namespace quartet
