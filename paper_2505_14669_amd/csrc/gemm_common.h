// Pieces shared by the matrix-core GEMM kernels: buffer resources, LDS-direct loads and the epilogue
// that takes a wave's accumulator tile through LDS to full-line stores.
#pragma once
#include "device_common.h"

namespace quartet {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Raw buffer resource over [base, base + bytes): loads past the end return zero, which is how ragged
// tile edges are handled without per-load predicates.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset no resource here reaches

// Plain epilogue of a kernel whose ring is free when it ends (the MXFP8 twin): the wave's accumulator tile goes through
// LDS one 32-column slice at a time and comes back with 8 consecutive lanes holding the 32 columns of one row (4 each):
// a store instruction then writes 8 whole 128-byte lines.  wbuf: this wave's LDS scratch of TM*32 rows x kEpiStride floats.
constexpr uint32_t kEpiStride = 32;   // floats per LDS row, no padding: the LDS has 64 banks and serves a 16-byte read 16 lanes (two rows here) at a time, so neighbouring rows must sit 32 banks apart (counters: every read took twice its cycles with rows of 36 or 40 floats)

template <int TM, int TN, bool OUT_BF16>
__device__ __forceinline__ void store_tile(v16f (&acc)[TM][TN], float* wbuf, void* d, uint32_t ldd, float alpha,
                                           uint32_t row_base, uint32_t col_base, uint32_t m, uint32_t n, uint32_t lane) {
    constexpr uint32_t ITERS = TM * 4;   // 8 rows per pass
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
    const uint32_t sub = lane >> 3, c = lane & 7u;
    const bool wide = (ldd & 3u) == 0u;   // every 4-column chunk starts 16-byte (fp32) / 8-byte (bf16) aligned
#pragma unroll
    for (uint32_t j = 0; j < TN; ++j) {
        const uint32_t gcol = col_base + j * 32u;
#pragma unroll
        for (uint32_t i = 0; i < TM; ++i)
#pragma unroll
            for (uint32_t r = 0; r < 16; ++r)
                wbuf[(i * 32u + (r >> 2) * 8u + lhalf * 4u + (r & 3u)) * kEpiStride + lrow] = acc[i][j][r];
        float4 slice[ITERS];   // all reads in flight before the first use: one wave per SIMD hides no LDS latency
#pragma unroll
        for (uint32_t it = 0; it < ITERS; ++it)
            slice[it] = *reinterpret_cast<const float4*>(&wbuf[(it * 8u + sub) * kEpiStride + 4u * c]);
#pragma unroll
        for (uint32_t it = 0; it < ITERS; ++it) {
            const uint32_t grow = row_base + it * 8u + sub;
            const float v0 = slice[it].x * alpha, v1 = slice[it].y * alpha, v2 = slice[it].z * alpha, v3 = slice[it].w * alpha;
            if (grow >= m) continue;
            const uint32_t col = gcol + 4u * c;
            const size_t at = (size_t)grow * ldd + col;
            if (OUT_BF16) {
                uint16_t* dst = static_cast<uint16_t*>(d) + at;
                const uint32_t h0 = f32_to_bf16_rne(v0), h1 = f32_to_bf16_rne(v1), h2 = f32_to_bf16_rne(v2), h3 = f32_to_bf16_rne(v3);
                if (wide && col + 4u <= n) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
                } else {
                    if (col < n) dst[0] = (uint16_t)h0;
                    if (col + 1u < n) dst[1] = (uint16_t)h1;
                    if (col + 2u < n) dst[2] = (uint16_t)h2;
                    if (col + 3u < n) dst[3] = (uint16_t)h3;
                }
            } else {
                float* dst = static_cast<float*>(d) + at;
                if (wide && col + 4u <= n) {
                    *reinterpret_cast<float4*>(dst) = make_float4(v0, v1, v2, v3);
                } else {
                    if (col < n) dst[0] = v0;
                    if (col + 1u < n) dst[1] = v1;
                    if (col + 2u < n) dst[2] = v2;
                    if (col + 3u < n) dst[3] = v3;
                }
            }
        }
    }
}

// One butterfly stage between a lane and its DPP partner for the four values of a chunk, one instruction per value: both
// lanes form partner * t + own (t = +-1, so the fused multiply-add rounds exactly like the addition): t = +1 in the lower
// lane gives a + b, t = -1 in the upper lane gives -(a - b).  A lane's values therefore carry the sign (-1)^(number of
// stages in which it was the upper one); the partners of every stage have been upper equally often before it, so the signs
// cancel inside each stage, and the normalization constant takes the final sign back (epilogue_norm).  Rounding is symmetric
// in sign: the bits are those of a + b and a - b.
// The instruction is written out (the compiler keeps a separate lane move in front of a fused multiply-add).  A DPP
// operand must not be read in the two issue slots after a vector instruction wrote it: hence the s_nop in front, and the
// three stages of the four values in one block, where every value is read four instructions after it was written.
#define QUARTET_DPP_TAIL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
#define QUARTET_BUTTERFLY_STAGE(CTRL_TEXT, T)                           \
    "v_fmac_f32_dpp %0, %0, " T " " CTRL_TEXT QUARTET_DPP_TAIL            \
    "v_fmac_f32_dpp %1, %1, " T " " CTRL_TEXT QUARTET_DPP_TAIL            \
    "v_fmac_f32_dpp %2, %2, " T " " CTRL_TEXT QUARTET_DPP_TAIL            \
    "v_fmac_f32_dpp %3, %3, " T " " CTRL_TEXT QUARTET_DPP_TAIL
// strides 4, 8, 16 of a 32-column slice held as four values in each of eight lanes: partners lane ^ 1, lane ^ 2, 7 - lane.
// volatile: the block reads other lanes, so it must stay where all lanes of a row group are active (not be moved into the
// predicated store that uses its results).
#define QUARTET_BUTTERFLIES_ACROSS(v0, v1, v2, v3, t4, t8, t16)                        \
    asm volatile("s_nop 1\n\t"                                                              \
        QUARTET_BUTTERFLY_STAGE("quad_perm:[1,0,3,2]", "%4")                            \
        QUARTET_BUTTERFLY_STAGE("quad_perm:[2,3,0,1]", "%5")                            \
        QUARTET_BUTTERFLY_STAGE("row_half_mirror", "%6")                                \
        : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3) : "v"(t4), "v"(t8), "v"(t16))
// v * (+-norm) with the lane's sign taken back; the added +0 turns a zero of either sign into +0, which is what sums and
// differences of the unsigned values give (x - x = +0, and no -0 enters: masked elements and empty sums are +0).
__device__ __forceinline__ float epilogue_norm(float v, float signed_norm) { return __builtin_fmaf(v, signed_norm, 0.0f); }

// Epilogue of the streaming kernels: the wave's accumulator tile leaves in passes of 8 rows x TN*32 columns through a
// scratch of the wave's own (outside the ring, so the ring keeps streaming the next tile); every store instruction writes
// 8 whole 128-byte lines.  With FUSED the gradient epilogue of Algorithm 1 Backward, D = alpha * H_along_n(acc . M), is
// applied on the way: mask select, the stages that combine whole 32-column groups and butterflies of stride 1 and 2 inside
// the lane, strides 4, 8, 16 between the 8 lanes that hold a row's slice (QUARTET_BUTTERFLIES_ACROSS: lane i holds 4-column
// chunk i ^ (i & 4 ? 3 : 0), which makes the partners lane ^ 1, lane ^ 2 and 7 - lane, all reachable by DPP), the
// normalization, then the scale: the same fp32 operations in the same order as the stand-alone epilogue kernel.
// Row 4*lhalf + e of a pass comes from register 4*qd + e of the four accumulators of tile row i; a lane reads
// back chunk c (4 columns) of all four 32-column slices of row `sub`, so Hadamard blocks of 32, 64 and 128 columns
// are handled alike (group-combining stages inside the lane, then the 32-point stages of each slice).
// LDS image: row r at r * TN*32 floats with its slices j stored at position j ^ f(r), f(r) = (r ^ r/4) & 1: the LDS has
// 64 banks and serves a 16-byte read 16 lanes at a time -- rows 2a and 2a+1 here, which f puts into different bank halves
// (counters: without it every read took twice its cycles); rows r and r+4, the two half-waves of a write, differ too.
template <int TM, int TN, bool OUT_BF16, bool FUSED, bool FULL>
__device__ __forceinline__ void store_tile_rows8(v16f (&acc)[TM][TN], float* wbuf, void* d, uint32_t ldd,
                                                 const uint32_t* mask, float alpha, uint32_t row_base,
                                                 uint32_t col_base, uint32_t m, uint32_t n, uint32_t lane, uint32_t nb) {
    static_assert(TN == 2 || TN == 4, "the slice swap of rows 4..7 pairs the slices up");
    constexpr uint32_t PASSES = TM * 4, W = TN * 32;
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
    const uint32_t sub = lane >> 3, c = (lane & 7u) ^ ((lane & 4u) ? 3u : 0u);
    const float up4 = (c & 1u) ? -1.0f : 1.0f, up8 = (c & 2u) ? -1.0f : 1.0f, up16 = (c & 4u) ? -1.0f : 1.0f;
    const float norm = ((c ^ (c >> 1) ^ (c >> 2)) & 1u) ? -block_norm(nb) : block_norm(nb);
    const bool wide = FULL || (ldd & 3u) == 0u;
    const uint32_t mask_ld = n >> 5;
    float* wr = wbuf + lhalf * 4u * W + lrow;          // + e*W + ((j ^ f(4 lhalf + e)) * 32)
    const float* rd = wbuf + sub * W + 4u * c;         // + ((j ^ f(sub)) * 32)
    const uint32_t rswz = (sub ^ (sub >> 2)) & 1u;
    uint32_t mw[PASSES][TN];
    if (FUSED) {
        const bool mvec = FULL && TN == 4 && (mask_ld & 3u) == 0u && (reinterpret_cast<uintptr_t>(mask) & 15u) == 0u;   // wave-uniform
#pragma unroll
        for (uint32_t p = 0; p < PASSES; ++p) {
            const uint32_t grow = row_base + p * 8u + sub;
            if (mvec) {
                const uint4 w4 = *reinterpret_cast<const uint4*>(&mask[(size_t)grow * mask_ld + (col_base >> 5)]);
                mw[p][0] = w4.x; mw[p][1] = w4.y; mw[p][2] = w4.z; mw[p][3] = w4.w;
            } else {
#pragma unroll
                for (uint32_t j = 0; j < TN; ++j) {
                    const uint32_t gcol = col_base + j * 32u;
                    if (FULL) mw[p][j] = mask[(size_t)grow * mask_ld + (gcol >> 5)];
                    else mw[p][j] = (mask && grow < m && gcol < n) ? mask[(size_t)grow * mask_ld + (gcol >> 5)] : 0xFFFFFFFFu;
                }
            }
        }
    }
#define ROWS8_WRITE(P)                                                                                  \
    _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j)                                                 \
        _Pragma("unroll") for (uint32_t e = 0; e < 4; ++e)                                              \
            wr[e * W + ((j ^ ((e & 1u) ^ lhalf)) * 32u)] = acc[(P) >> 2][j][((P) & 3u) * 4u + e];
    ROWS8_WRITE(0u)
#pragma unroll
    for (uint32_t p = 0; p < PASSES; ++p) {
        float4 sl[TN];
#pragma unroll
        for (uint32_t j = 0; j < TN; ++j) sl[j] = *reinterpret_cast<const float4*>(&rd[(j ^ rswz) * 32u]);
        if (p + 1u < PASSES) { ROWS8_WRITE(p + 1u) }     // behind the reads in the wave's LDS queue: LDS operations of a wave run in order
        const uint32_t grow = row_base + p * 8u + sub;
        float vv[TN][4];
#pragma unroll
        for (uint32_t j = 0; j < TN; ++j) {
            vv[j][0] = sl[j].x; vv[j][1] = sl[j].y; vv[j][2] = sl[j].z; vv[j][3] = sl[j].w;
            if (FUSED) {
                const int32_t bits = (int32_t)(mw[p][j] >> (4u * c));
#pragma unroll
                for (uint32_t e = 0; e < 4; ++e)
                    vv[j][e] = __uint_as_float(__float_as_uint(vv[j][e]) & (uint32_t)((bits << (31 - (int)e)) >> 31));
            }
        }
        if (FUSED && nb >= 2u) {
#pragma unroll
            for (uint32_t j = 0; j + 1u < TN; j += 2)
#pragma unroll
                for (uint32_t e = 0; e < 4; ++e) {
                    const float a = vv[j][e], b = vv[j + 1][e];
                    vv[j][e] = a + b;
                    vv[j + 1][e] = a - b;
                }
        }
        if (FUSED && nb >= 4u && TN >= 4) {
#pragma unroll
            for (uint32_t j = 0; j < 2; ++j)
#pragma unroll
                for (uint32_t e = 0; e < 4; ++e) {
                    const float a = vv[j][e], b = vv[(j + 2u) % TN][e];
                    vv[j][e] = a + b;
                    vv[(j + 2u) % TN][e] = a - b;
                }
        }
#pragma unroll
        for (uint32_t j = 0; j < TN; ++j) {
            const uint32_t gcol = col_base + j * 32u;
            float v0 = vv[j][0], v1 = vv[j][1], v2 = vv[j][2], v3 = vv[j][3];
            if (FUSED) {
                const float a0 = v0 + v1, a1 = v0 - v1, a2 = v2 + v3, a3 = v2 - v3;
                v0 = a0 + a2; v2 = a0 - a2; v1 = a1 + a3; v3 = a1 - a3;
                QUARTET_BUTTERFLIES_ACROSS(v0, v1, v2, v3, up4, up8, up16);
                v0 = epilogue_norm(v0, norm); v1 = epilogue_norm(v1, norm); v2 = epilogue_norm(v2, norm); v3 = epilogue_norm(v3, norm);
            }
            v0 = v0 * alpha; v1 = v1 * alpha; v2 = v2 * alpha; v3 = v3 * alpha;
            if (!FULL && grow >= m) continue;
            const uint32_t col = gcol + 4u * c;
            const size_t at = (size_t)grow * ldd + col;
            if (OUT_BF16) {
                uint16_t* dst = static_cast<uint16_t*>(d) + at;
                const uint32_t h0 = f32_to_bf16_rne(v0), h1 = f32_to_bf16_rne(v1), h2 = f32_to_bf16_rne(v2), h3 = f32_to_bf16_rne(v3);
                if (FULL || (wide && col + 4u <= n)) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
                } else {
                    if (col < n) dst[0] = (uint16_t)h0;
                    if (col + 1u < n) dst[1] = (uint16_t)h1;
                    if (col + 2u < n) dst[2] = (uint16_t)h2;
                    if (col + 3u < n) dst[3] = (uint16_t)h3;
                }
            } else {
                float* dst = static_cast<float*>(d) + at;
                if (FULL || (wide && col + 4u <= n)) {
                    *reinterpret_cast<float4*>(dst) = make_float4(v0, v1, v2, v3);
                } else {
                    if (col < n) dst[0] = v0;
                    if (col + 1u < n) dst[1] = v1;
                    if (col + 2u < n) dst[2] = v2;
                    if (col + 3u < n) dst[3] = v3;
                }
            }
        }
    }
#undef ROWS8_WRITE
}


// Depth of the LDS ring of the large-tile kernels.
constexpr uint32_t kRing = 4;

typedef int v4i_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ v4i_t make_rsrc_words(const void* base, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    v4i_t r = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), (int)bytes, 0x00020000};
    return r;
}

// 16 bytes per lane from the buffer resource at byte offset voff (past the end: zeros) to LDS byte
// address lds_base + 16 * lane.  lds_base must be wave-uniform.  Completion is counted by vmcnt.
__device__ __forceinline__ void lds_direct_load16(v4i_t rsrc, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc) : "memory");
}

}  // namespace quartet
