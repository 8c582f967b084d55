// Fused Hadamard + MXFP4 quantizer kernels for gfx950 (Algorithm 1, "Stage 1" of Section 4.4).
//
// One lane owns one group of 32 values end to end: the five butterfly stages, the group
// reduction (sum of squares or absmax), the scale and the 32 codes all stay in that lane's
// registers, so nothing crosses lanes and the fp32 operation order is fixed (Hadamard blocks of
// 64, 128 or 256 elements add the stages that combine whole groups in front: lane exchanges in row
// mode, a butterfly tree over the block's source-row groups in the transposed kernels).  HBM traffic
// is made wave-coalesced on both sides by staging through LDS:
//   row mode        : a wave loads 4 KB (64 groups) with 16-byte lane-contiguous loads, swizzles it
//                     through LDS so each lane gets its own 64 bytes; codes leave as one 16-byte
//                     store per lane.
//   transposed mode : a block owns 256 source rows x 128 source columns; lanes read 2 adjacent
//                     columns per row (4-byte loads, 256 B per wave row), and the 8 groups of codes
//                     of each output row are gathered in LDS and written as full 128-byte lines.
#include "device_common.h"
#include "launchers.h"

namespace quartet {

// Eight values -> eight E2M1 codes in one dword: round-to-nearest-even of v/scale (scale a power
// of two), saturating at +-6, element j in bits [4j, 4j+4).
__device__ __forceinline__ uint32_t rtn_pack8(const float* v, float scale) {
    uint32_t w = 0u;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[0], v[1], scale, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[2], v[3], scale, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[4], v[5], scale, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[6], v[7], scale, 3);
    return w;
}

// Encode one rotated group held in v[]: scale, codes, mask.  q_base = (linear output position of
// element 0)/16 is the Philox call index of the group's first 16 elements.
template <int MODE>
__device__ __forceinline__ void encode_group(float (&v)[32], const SrParams& p, uint64_t q_base,
                                             uint4& codes, uint32_t& scale_byte, uint32_t& mask_word);

__device__ __forceinline__ void flip_signs(float (&v)[32], uint32_t sign_word) {
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = u2f(f2u(v[i]) ^ (((sign_word >> i) & 1u) << 31));
}

// Quantize one group held in v[] (not yet rotated), Hadamard block = the group.  FLIPPED: the caller has applied the
// sign vector of the randomized rotation already (where it is cheaper: while unpacking, or on the codes before decoding).
template <int MODE, bool FLIPPED = false>
__device__ __forceinline__ void quantize_group(float (&v)[32], const SrParams& p, uint64_t q_base,
                                               uint4& codes, uint32_t& scale_byte, uint32_t& mask_word) {
    if (MODE != kFwd && !FLIPPED) flip_signs(v, p.sign_word);
    fwht32(v);
    encode_group<MODE>(v, p, q_base, codes, scale_byte, mask_word);
}

// The same when the Hadamard block spans p.nb groups held by consecutive lanes (lane % nb = the
// group's place in its block): signs, the group-combining stages across lanes, the stages inside the
// group, one normalization.  Every lane of the wave must call it.
template <int MODE>
__device__ __forceinline__ void quantize_group_lanes(float (&v)[32], const SrParams& p, uint32_t lane, uint64_t q_base,
                                                     uint4& codes, uint32_t& scale_byte, uint32_t& mask_word) {
    if (MODE != kFwd) {
        uint32_t sw = p.sign_words[0];
#pragma unroll
        for (uint32_t j = 1; j < 8; ++j) sw = ((lane & (p.nb - 1u)) == j) ? p.sign_words[j] : sw;
        flip_signs(v, sw);
    }
    cross_lane_stages(v, lane, p.nb);
    fwht32_unscaled(v);
    const float c = block_norm_signed(p.nb, lane);
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = __builtin_fmaf(v[i], c, 0.0f);
    encode_group<MODE>(v, p, q_base, codes, scale_byte, mask_word);
}

template <int MODE>
__device__ __forceinline__ void encode_group(float (&v)[32], const SrParams& p, uint64_t q_base,
                                             uint4& codes, uint32_t& scale_byte, uint32_t& mask_word) {
    uint32_t c[4] = {0u, 0u, 0u, 0u};
    if (MODE == kFwd) {
        // QuEST: scale from the group RMS, round to nearest, remember what clipped
        float t[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) t[i] = v[i] * v[i];
#pragma unroll
        for (int n = 16; n >= 1; n >>= 1) {
#pragma unroll
            for (int i = 0; i < n; ++i) t[i] = t[2 * i] + t[2 * i + 1];
        }
        uint32_t E = (f2u(t[0]) >> 23) & 0xFFu;
        int e = (E == 0u) ? 0 : (((int)E - 133) >> 1);   // floor((log2 ss - 6) / 2)
        uint32_t b = (uint32_t)(e + 127);
        float scale = u2f(b << 23);                        // 2^e
        float thr = u2f(0x40C00000u + ((uint32_t)e << 23)); // 6 * 2^e
        uint32_t m = 0u;
#pragma unroll
        for (int i = 31; i >= 0; --i) m = (m << 1) | (__builtin_fabsf(v[i]) <= thr ? 1u : 0u);
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i] = rtn_pack8(&v[8 * i], scale);
        scale_byte = b;
        mask_word = m;
    } else {
        // AbsMax power-of-two scale, 3/4 range matching, RTN or SR (nothing clips)
        float mx = 0.0f;
#pragma unroll
        for (int i = 0; i < 32; ++i) mx = __builtin_fmaxf(mx, __builtin_fabsf(v[i]));
        uint32_t E = (f2u(mx) >> 23) & 0xFFu;
        uint32_t b = (E == 0u) ? 127u : (E >= 2u ? E - 2u : 0u);
        float mult = u2f((254u - b) << 23) * 0.75f;        // 3/4 * 2^-e, exact
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = v[i] * mult;
        if (MODE == kBwdRtn) {
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] = rtn_pack8(&v[8 * i], 1.0f);
        } else {
#pragma unroll
            for (int call = 0; call < 2; ++call) {
                uint64_t q = q_base + (uint64_t)call;
                uint32_t w[4];
                philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), p.stream_id, 0u, p.key0, p.key1, w);
                c[2 * call] = sr_pack8(&v[16 * call], w[0], w[1]);
                c[2 * call + 1] = sr_pack8(&v[16 * call + 8], w[2], w[3]);
            }
        }
        scale_byte = b;
        mask_word = 0xFFFFFFFFu;
    }
    codes = make_uint4(c[0], c[1], c[2], c[3]);
}

// Sign bit of element i of the randomized rotation's sign vector as a float's sign bit (wave-uniform: scalar arithmetic).
__device__ __forceinline__ uint32_t sign_bit(uint32_t sign_word, uint32_t i) { return ((sign_word >> i) & 1u) << 31; }

// Eight bf16 values (elements first .. first+7 of a group) to fp32 with the sign vector applied on the way.  An even
// element is x << 16 plus its sign bit: adding 0x80000000 flips the top bit, and shift-and-add is one instruction where
// shift and XOR are two; an odd element is one three-input bit operation either way.
__device__ __forceinline__ void unpack_bf16x8_signed(const uint4& q, float* v, uint32_t sign_word, uint32_t first) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        v[2 * j] = u2f((w[j] << 16) + sign_bit(sign_word, first + 2u * j));
        v[2 * j + 1] = u2f((w[j] & 0xFFFF0000u) ^ sign_bit(sign_word, first + 2u * j + 1u));
    }
}

__device__ __forceinline__ void unpack_bf16x8(const uint4& q, float* v) {
    v[0] = u2f(q.x << 16); v[1] = u2f(q.x & 0xFFFF0000u);
    v[2] = u2f(q.y << 16); v[3] = u2f(q.y & 0xFFFF0000u);
    v[4] = u2f(q.z << 16); v[5] = u2f(q.z & 0xFFFF0000u);
    v[6] = u2f(q.w << 16); v[7] = u2f(q.w & 0xFFFF0000u);
}

// ------------------------------------------------------------------ row mode
// Block = 8 rows x 32 groups (four 256-element K-quads, 2 KB of bf16 per row).  Wave w owns rows
// 2w, 2w+1; lane l the group l%32 of row l/32.  Loads are lane-contiguous 16-byte chunks, swizzled
// through LDS so each lane ends up with its own group's 64 bytes.  Codes leave as 512 contiguous
// bytes per row, mask words as 128; the 256 scale bytes of the block are exchanged through LDS and
// leave as whole 32-byte runs of the scale tiles (8 rows x one dword), never as single bytes.
// BIG: the Hadamard block spans p.nb = 2, 4 or 8 groups; they sit in consecutive lanes (a row's groups
// start at a multiple of 8 in every block), so the group-combining stages are lane exchanges.
// bid: the block's number in its matrix; stage (16 KB), s_scale (256 B): the block's LDS
template <int MODE, bool MASK, bool BIG>
__device__ __forceinline__ void quant_row_tile(const uint16_t* __restrict__ x, uint32_t rows, uint32_t gk, int64_t ldx,
                                               uint4* __restrict__ codes, uint8_t* __restrict__ scales, uint32_t* __restrict__ mask,
                                               const SrParams& p, uint32_t k_blocks, FastDiv div_k_blocks, uint32_t bid,
                                               uint4 (*stage)[256], uint32_t* s_scale) {
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    // consecutive blocks walk along K inside the same 8 rows, so the blocks in flight cover one
    // contiguous stretch of the input
    const uint32_t row_set = fast_div(bid, div_k_blocks);
    const uint32_t row0 = row_set * 8u, kq0 = (bid - row_set * k_blocks) * 4u, kqs = (gk + 7u) >> 3;
    // The block's rows through a buffer resource that ends with the last element of its last row:
    // rows past the matrix read as zeros without a predicate.  Groups past k inside a row read
    // whatever lies there (the row's padding or the next row); their results are never stored.
    const uint32_t rows_here = (rows - row0) < 8u ? (rows - row0) : 8u;
    const __amdgpu_buffer_rsrc_t res_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(x + (size_t)row0 * ldx), 0, (int)(((rows_here - 1u) * (uint32_t)ldx + gk * 32u) * 2u), 0x00020000);
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        uint32_t c = 64u * j + lane;                       // 16-byte chunk inside the wave's 2 rows x 2 KB
        const uint32_t voff = ((wave * 2u + (c >> 7)) * (uint32_t)ldx + kq0 * 256u + (c & 127u) * 8u) * 2u;
        v4u_t q = __builtin_amdgcn_raw_buffer_load_b128(res_x, (int)voff, 0, 2 /* non-temporal */);
        stage[wave][(c & ~3u) | ((c & 3u) ^ ((c >> 4) & 3u))] = make_uint4(q.x, q.y, q.z, q.w);
    }
    __syncthreads();
    float v[32];
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        uint4 q = stage[wave][4u * lane + (j ^ ((lane >> 2) & 3u))];
        if (MODE != kFwd && !BIG) unpack_bf16x8_signed(q, &v[8 * j], p.sign_word, 8u * j);
        else unpack_bf16x8(q, &v[8 * j]);
    }
    const uint32_t row_local = wave * 2u + (lane >> 5), gi = lane & 31u;
    const uint32_t row = row0 + row_local, g = kq0 * 8u + gi;
    uint4 out;
    uint32_t sb, mw;
    if (BIG) quantize_group_lanes<MODE>(v, p, lane, ((uint64_t)row * gk + g) * 2u, out, sb, mw);
    else quantize_group<MODE, true>(v, p, ((uint64_t)row * gk + g) * 2u, out, sb, mw);
    // scale byte of (row, group gi) -> position of the tiled layout inside the block's 256 bytes:
    // [K-quad gi/8][h = gi%2][row_local][p = (gi%8)/2]
    reinterpret_cast<uint8_t*>(s_scale)[(((gi >> 3) * 2u + (gi & 1u)) * 8u + row_local) * 4u + ((gi & 7u) >> 1)] = (uint8_t)sb;
    if (row < rows && g < gk) {
        const size_t gidx = (size_t)row * gk + g;
        store_stream16(&codes[gidx], out);
        if (MASK) store_stream4(&mask[gidx], mw);
    }
    __syncthreads();
    if (threadIdx.x < 64u) {
        const uint32_t t = threadIdx.x, kql = t >> 4, h = (t >> 3) & 1u, rl = t & 7u;
        const uint32_t r = row0 + rl, kq = kq0 + kql;
        if (r < rows && kq * 8u + h < gk) {
            uint8_t* dst = scales + scale_tile_offset(r, kq * 8u + h, kqs);   // dword of (row, h) in tile kq
            const uint32_t w = s_scale[t];
            if (kq * 8u + 8u <= gk) {
                *reinterpret_cast<uint32_t*>(dst) = w;
            } else {                                         // ragged last K-quad: only the bytes that exist
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q)
                    if (kq * 8u + 2u * q + h < gk) dst[q] = (uint8_t)(w >> (8u * q));
            }
        }
    }
}

template <int MODE, bool MASK, bool BIG>
__global__ void __launch_bounds__(256)
quant_row_kernel(const uint16_t* __restrict__ x, uint32_t rows, uint32_t gk, int64_t ldx,
                 uint4* __restrict__ codes, uint8_t* __restrict__ scales, uint32_t* __restrict__ mask,
                 SrParams p, uint32_t k_blocks, FastDiv div_k_blocks) {
    __shared__ uint4 stage[4][256];
    __shared__ uint32_t s_scale[64];
    quant_row_tile<MODE, MASK, BIG>(x, rows, gk, ldx, codes, scales, mask, p, k_blocks, div_k_blocks, blockIdx.x, stage, s_scale);
}

// Two matrices with the same inner dimension in one launch (Algorithm 1 Forward quantizes X and W, and neither depends
// on the other): blocks [0, split) work on the first, the rest on the second.  A weight-sized matrix alone fills the chip
// for a few microseconds only, most of it ramp-up and drain; behind the activations' blocks it costs its bytes.
struct RowMatrix {
    const uint16_t* x;
    uint32_t rows;
    int64_t ldx;
    uint4* codes;
    uint8_t* scales;
    uint32_t* mask;
};

template <int MODE, bool MASK>
__global__ void __launch_bounds__(256)
quant_row_pair_kernel(RowMatrix a, RowMatrix b, uint32_t split, uint32_t gk, SrParams p, uint32_t k_blocks, FastDiv div_k_blocks) {
    __shared__ uint4 stage[4][256];
    __shared__ uint32_t s_scale[64];
    const bool second = blockIdx.x >= split;
    const RowMatrix& m = second ? b : a;
    quant_row_tile<MODE, MASK, false>(m.x, m.rows, gk, m.ldx, m.codes, m.scales, m.mask, p, k_blocks, div_k_blocks,
                                      second ? blockIdx.x - split : blockIdx.x, stage, s_scale);
}

// Store phase of the transposed kernels: the tile's codes, scale bytes and mask words gathered in LDS
// ([local column][group], codes with a 16-byte slot swizzle; columns 16..31 of every 32 swap places in pairs, which
// puts the 16 lanes of a 16-byte LDS access on the 64 banks' 16 different slots) leave as full 128-byte lines of codes,
// 32-byte runs of mask words and whole dwords of the scale tiles.
template <bool MASK>
__device__ __forceinline__ void transposed_store_tile(const uint4* s_codes, const uint8_t* s_scales, const uint32_t* s_mask,
                                                      uint32_t col0, uint32_t grp0, uint32_t rows, uint32_t gk, uint32_t k,
                                                      uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                                      uint32_t* __restrict__ mask) {
    // full 128-byte lines of codes: 8 lanes per output row
#pragma unroll
    for (uint32_t j = 0; j < 4; ++j) {
        uint32_t id = threadIdx.x + 256u * j;
        uint32_t lc = id >> 3, part = id & 7u;
        uint32_t r = col0 + lc, grp = grp0 + part;
        if (r < rows && grp < gk) {
            uint4 q = s_codes[(lc ^ ((lc >> 4) & 1u)) * 8u + (part ^ ((lc >> 1) & 7u))];
            store_stream16(codes + (size_t)r * (k >> 1) + (size_t)grp * 16u, q);
        }
    }
    if (MASK) {
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            uint32_t id = threadIdx.x + 256u * j;
            uint32_t lc = id >> 3, part = id & 7u;
            uint32_t r = col0 + lc, grp = grp0 + part;
            if (r < rows && grp < gk) mask[(size_t)r * gk + grp] = s_mask[lc * 8u + part];
        }
    }
    // scales: the block's 8 groups are one K-quad, so each 32-row block of the tile is one 256-byte
    // scale tile; thread t writes dword t%64 of tile t/64 (bytes = groups h, 2+h, 4+h, 6+h of its row)
    const uint32_t t = threadIdx.x, lc = (t >> 6) * 32u + (t & 31u), h = (t >> 5) & 1u;
    const uint32_t r = col0 + lc;
    if (r < rows) {
        uint32_t w = 0u;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) w |= (uint32_t)s_scales[lc * 8u + 2u * q + h] << (8u * q);
        const uint32_t kq = (gk + 7u) >> 3;
        uint32_t* dst = reinterpret_cast<uint32_t*>(scales + scale_tile_offset(r, grp0 + h, kq));
        if (grp0 + 6u + h < gk) {
            *dst = w;
        } else {
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (grp0 + 2u * q + h < gk) reinterpret_cast<uint8_t*>(dst)[q] = (uint8_t)(w >> (8u * q));
        }
    }
}

// ------------------------------------------------------------------ transposed mode, bf16 source
// Logical A[rows x k] = S^T where the source S is bf16 [k x ldx].
// Block tile: 8 groups (256 source rows, one K-quad of the output) x 128 source columns; wave w owns
// groups 2w, 2w+1; lane l owns columns 2l, 2l+1.  Blocks are numbered K-quad first: the blocks that
// run at the same time then write neighbouring 128-byte lines of the same output rows (measured 10 %
// faster than column-tile first, where every block's lines lie a whole output row apart).  The callers
// rotate the column tile by the K-quad (transposed_column_tile): with a dense source whose row pitch is a
// multiple of a few KB, the blocks in flight would otherwise all read the same 4 KB-wide stretch of
// columns of every row, which the memory channels serve unevenly (measured: 5-9 % slower; a source
// with 128 bytes of padding per row does not show it).
// bx, by: the block's K-quad and column tile; s_codes (16 KB), s_scales (1 KB), s_mask (4 KB): the block's LDS
template <int MODE, bool MASK>
__device__ __forceinline__ void quant_transposed_tile(const uint16_t* __restrict__ src,
                                                      uint32_t rows, uint32_t k, int64_t ldx, uint8_t* __restrict__ codes,
                                                      uint8_t* __restrict__ scales, uint32_t* __restrict__ mask,
                                                      const SrParams& p, uint32_t bx, uint32_t by,
                                                      uint4* s_codes, uint8_t* s_scales, uint32_t* s_mask) {
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63u;
    const uint32_t gk = k >> 5;
    const uint32_t col0 = by * 128u;
    const uint32_t grp0 = bx * 8u;
    const uint32_t col = col0 + 2u * lane;                // even; rows is even, so col+1 < rows too
    // the block's corner of the source through a buffer resource that ends with the last column of the
    // last source row
    const uint32_t src_rows = (k - grp0 * 32u) < 256u ? (k - grp0 * 32u) : 256u;
    const uint32_t src_cols = (rows - col0) < 128u ? (rows - col0) : 128u;
    const __amdgpu_buffer_rsrc_t res_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(src + (size_t)grp0 * 32u * ldx + col0), 0,
        (int)(((src_rows - 1u) * (uint32_t)ldx + src_cols) * 2u), 0x00020000);

    // all 64 loads of the wave's two groups go out before any arithmetic: the second group's data
    // arrives while the first is rotated and quantized.  Rows past k read as zeros without a predicate
    // (the wave-uniform row offset rides in the scalar offset and takes part in the range check);
    // columns past `rows` inside a source row read whatever lies there, their results are never stored.
    uint32_t raw[2][32];
#pragma unroll
    for (uint32_t rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (uint32_t i = 0; i < 32; ++i)
            raw[rb][i] = __builtin_amdgcn_raw_buffer_load_b32(
                res_x, (int)(4u * lane), (int)(((2u * wave + rb) * 32u + i) * (uint32_t)ldx * 2u), 2 /* non-temporal */);
    }
#pragma unroll
    for (uint32_t rb = 0; rb < 2; ++rb) {
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t gl = 2u * wave + rb;               // group inside the block tile
        const uint32_t grp = grp0 + gl;
        const uint32_t sw = lane & 7u;                    // 16-byte slot swizzle against bank conflicts
#pragma unroll
        for (uint32_t c = 0; c < 2; ++c) {
            float v[32];
#pragma unroll
            for (uint32_t i = 0; i < 32; ++i) {       // with the sign vector applied on the way (forward: sign word 0 in p)
                const uint32_t sbit = MODE != kFwd ? sign_bit(p.sign_word, i) : 0u;
                v[i] = c ? u2f((raw[rb][i] & 0xFFFF0000u) ^ sbit) : u2f((raw[rb][i] << 16) + sbit);
            }
            uint4 q;
            uint32_t sb, m;
            // output position of element 0 of the group: row*k + grp*32, divided by 16
            quantize_group<MODE, true>(v, p, ((uint64_t)(col + c) * k + grp * 32u) >> 4, q, sb, m);
            const uint32_t lc = 2u * lane + c;            // local column
            s_codes[(lc ^ ((lc >> 4) & 1u)) * 8u + (gl ^ sw)] = q;
            s_scales[lc * 8u + gl] = (uint8_t)sb;
            if (MASK) s_mask[lc * 8u + gl] = m;
        }
    }
    __syncthreads();
    transposed_store_tile<MASK>(s_codes, s_scales, s_mask, col0, grp0, rows, gk, k, codes, scales, mask);
}

// Column tile of the block with K-quad bx and nominal column tile by, of n_ct column tiles (a bijection for every bx).
__device__ __forceinline__ uint32_t transposed_column_tile(uint32_t bx, uint32_t by, uint32_t n_ct) { return (by + bx) % n_ct; }

template <int MODE, bool MASK>
__global__ void __launch_bounds__(256, MODE == kBwdSr ? 3 : 4)
quant_transposed_kernel(const uint16_t* __restrict__ src,
                        uint32_t rows, uint32_t k, int64_t ldx, uint8_t* __restrict__ codes,
                        uint8_t* __restrict__ scales, uint32_t* __restrict__ mask, SrParams p) {
    __shared__ uint4 s_codes[128 * 8];
    __shared__ uint8_t s_scales[128 * 8];
    __shared__ uint32_t s_mask[128 * 8];
    quant_transposed_tile<MODE, MASK>(src, rows, k, ldx, codes, scales, mask, p, blockIdx.x,
                                      transposed_column_tile(blockIdx.x, blockIdx.y, gridDim.y), s_codes, s_scales, s_mask);
}

// The same tile for Hadamard blocks of NB = 2, 4 or 8 groups.  The groups of a block are whole source
// row groups, so the group-combining stages come first and work on raw values: for its two groups
// (places j, j+1 of one block) and each column of its pair a wave reads all NB groups of the block (the
// other waves of the block read the same lines: the extra reads are cache hits), folds them through the
// butterfly tree down to that place, and only then runs the 32-point stages.
template <int MODE, bool MASK, int NB>
__global__ void __launch_bounds__(256)
quant_transposed_block_kernel(const uint16_t* __restrict__ src, uint32_t rows, uint32_t k, int64_t ldx,
                              uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                              uint32_t* __restrict__ mask, SrParams p) {
    __shared__ uint4 s_codes[128 * 8];
    __shared__ uint8_t s_scales[128 * 8];
    __shared__ uint32_t s_mask[128 * 8];
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63u;
    const uint32_t gk = k >> 5;
    const uint32_t col0 = transposed_column_tile(blockIdx.x, blockIdx.y, gridDim.y) * 128u;
    const uint32_t grp0 = blockIdx.x * 8u;
    const uint32_t col = col0 + 2u * lane;
    const uint32_t src_rows = (k - grp0 * 32u) < 256u ? (k - grp0 * 32u) : 256u;
    const uint32_t src_cols = (rows - col0) < 128u ? (rows - col0) : 128u;
    const __amdgpu_buffer_rsrc_t res_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(src + (size_t)grp0 * 32u * ldx + col0), 0,
        (int)(((src_rows - 1u) * (uint32_t)ldx + src_cols) * 2u), 0x00020000);
    const uint32_t pitch = (uint32_t)ldx * 2u;
    const uint32_t gl0 = 2u * wave;                          // the wave's groups gl0, gl0+1 inside the tile
    const uint32_t jb = gl0 & ~((uint32_t)NB - 1u);           // first group of their Hadamard block
    const uint32_t j = gl0 - jb;                              // even place of gl0 in the block
    const uint32_t neg2 = (j & 2u) << 30, neg4 = (j & 4u) << 29;   // sign of the upper operand at the 64- and 128-stages
    const float norm = block_norm((uint32_t)NB);
    const uint32_t sw = lane & 7u;                            // 16-byte slot swizzle against bank conflicts
    // one output group of one column at a time: 32 results and four source rows of every group in flight keep the
    // kernel at four waves per SIMD (holding both groups of a column pair took all 512 registers of a lane)
#pragma unroll 1
    for (uint32_t pass = 0; pass < 4; ++pass) {
        const uint32_t c = pass & 1u, rb = pass >> 1;
        const uint32_t neg1 = rb << 31;                       // place j + rb: the 32-stage is a sum (rb = 0) or a difference
        // The loads do not depend on the pass, so the compiler lifts all 32 NB of them out of this loop and keeps
        // them in registers: good for NB = 2 and 4 (64 and 128 registers, every line read once), too much for
        // NB = 8 (all 512 registers of a lane, one wave per SIMD), where an offset it cannot see through keeps
        // them inside the pass.
        uint32_t lane_off = 4u * lane;
        if (NB > 4) asm volatile("" : "+v"(lane_off));
        float v[32];
#pragma unroll
        for (uint32_t i = 0; i < 32; ++i) {
            // at most four source rows of every group in flight: without the fence all 32 NB loads are
            // hoisted to the top and the kernel runs out of registers
            if ((i & 3u) == 0u) __builtin_amdgcn_sched_barrier(0);
            float x[NB];
#pragma unroll
            for (uint32_t jj = 0; jj < (uint32_t)NB; ++jj) {
                const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(res_x, (int)lane_off, (int)(((jb + jj) * 32u + i) * pitch), 0);
                uint32_t bits = c ? (w & 0xFFFF0000u) : (w << 16);
                if (MODE != kFwd) bits ^= ((p.sign_words[jj] >> i) & 1u) << 31;
                x[jj] = u2f(bits);
            }
            float y[NB / 2];
#pragma unroll
            for (uint32_t m = 0; m < (uint32_t)NB / 2u; ++m) y[m] = x[2 * m] + u2f(f2u(x[2 * m + 1]) ^ neg1);
            if (NB >= 4) {
#pragma unroll
                for (uint32_t m = 0; m < (uint32_t)NB / 4u; ++m) y[m] = y[2 * m] + u2f(f2u(y[2 * m + 1]) ^ neg2);
            }
            if (NB >= 8) y[0] = y[0] + u2f(f2u(y[1]) ^ neg4);
            v[i] = y[0];
        }
        fwht32_unscaled(v);
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = v[i] * norm;
        const uint32_t gl = gl0 + rb;
        uint4 q;
        uint32_t sbyte, m;
        encode_group<MODE>(v, p, ((uint64_t)(col + c) * k + (grp0 + gl) * 32u) >> 4, q, sbyte, m);
        const uint32_t lc = 2u * lane + c;
        s_codes[(lc ^ ((lc >> 4) & 1u)) * 8u + (gl ^ sw)] = q;
        s_scales[lc * 8u + gl] = (uint8_t)sbyte;
        if (MASK) s_mask[lc * 8u + gl] = m;
    }
    __syncthreads();
    transposed_store_tile<MASK>(s_codes, s_scales, s_mask, col0, grp0, rows, gk, k, codes, scales, mask);
}

// ------------------------------------------------------------------ MXFP4 source, other dimension
// Re-quantization of a saved MXFP4 tensor S [k x rows] along its other dimension (Algorithm 1
// Backward: the operands W_q^T and X_q^T).  A wave covers 256 source rows (one K-quad of the
// output) x 64 source columns (64 output rows) and works alone, without block barriers; four
// neighbouring waves make up a 256-column stretch (one scale tile wide).  Per output group (32
// source rows) a lane fetches 16 bytes of codes (32 columns of one source row; the four waves of a
// stretch together read whole 128-byte lines),
// decodes them exactly and writes the 32 values into the wave's LDS stage laid out
// [column][source row]; then lane c reads the 32 values of column c back, quantizes the group and
// keeps its 16 bytes of codes; the scale bytes collect in two registers that are, after the eighth
// group, exactly the two scale-tile dwords of the lane's output row.  Each lane then writes the 128
// contiguous bytes of codes of its row and its two scale dwords.
constexpr uint32_t kStageStride = 36;   // floats per column of the stage: 16-byte aligned, b128 reads conflict-free

// WPB = waves per block (the launcher uses 1: the waves of a 256-column stretch never cooperate, and blocks of one
// wave spread them over more CUs).
// The work of one wave: `wave` = its place in the 256-column stretch `quad`, kq = the K-quad of the output, stage = the
// wave's 64 x kStageStride floats of LDS.
template <int MODE>
__device__ __forceinline__ void requant_transposed_wave(const uint8_t* __restrict__ src_codes, const uint8_t* __restrict__ src_scales,
                                                        uint32_t rows, uint32_t k, uint8_t* __restrict__ codes,
                                                        uint8_t* __restrict__ scales, const SrParams& p,
                                                        uint32_t wave, uint32_t quad, uint32_t kq, float* stage) {
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t gk = k >> 5, okq = (k + 255u) >> 8;          // output groups per row, output K-quads
    const uint32_t half = rows >> 1, skq = (rows + 255u) >> 8;  // source row pitch in bytes, source K-quads
    const uint32_t c0 = quad * 256u + wave * 64u, grp0 = kq * 8u;
    // load role: source row rl of the group, 32-column chunk ch of the wave's 64 columns
    const uint32_t rl = lane >> 1, ch = lane & 1u, cg = wave * 2u + ch;   // cg: column group inside the source's K-quad
    // The block's corner of the source codes and the scale tiles below it through buffer resources that
    // end with the data: source rows past k read as zeros without predicates or branches.  Columns
    // past `rows` read whatever lies there; the output rows they feed are never stored.
    const uint32_t cb0 = quad * 256u;
    const uint32_t src_rows = (k - grp0 * 32u) < 256u ? (k - grp0 * 32u) : 256u;
    const uint32_t src_cols = (rows - cb0) < 256u ? (rows - cb0) : 256u;
    const __amdgpu_buffer_rsrc_t res_c = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(src_codes + (size_t)grp0 * 32u * half + (cb0 >> 1)), 0,
        (int)((src_rows - 1u) * half + (src_cols >> 1)), 0x00020000);
    // the 32 rows x 8 column groups of one step of the block are exactly one scale tile of the source
    const size_t tile0 = ((size_t)grp0 * skq + (cb0 >> 8)) * 256u;
    const __amdgpu_buffer_rsrc_t res_s = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(src_scales + tile0), 0, (int)((size_t)gk * skq * 256u - tile0), 0x00020000);
    const uint32_t code_off = rl * half + ((wave * 64u + 32u * ch) >> 1);
    const uint32_t scale_off = (((cg & 1u) << 5) + rl) * 4u + (cg >> 1);
    const uint32_t code_step = 32u * half, scale_step = skq * 256u;   // wave-uniform: they ride in the scalar offset
    const uint32_t wr = (rl + 16u * ch) & 31u;                  // rotated row slot: the 32 lanes of a write pass (16 source rows x 2 chunks) land on 32 different banks
    // quantize role: output row c0 + lane
    const uint32_t out_row = c0 + lane, rot = (16u * (lane >> 5)) & 31u;

    // sign of element rl of the rotation's sign vector as the sign bits of eight E2M1 codes (sign-magnitude: decoding
    // the flipped code gives the negated value exactly, zeros included)
    const uint32_t code_flip = (MODE != kFwd && ((p.sign_word >> rl) & 1u)) ? 0x88888888u : 0u;
    v4u_t cw = __builtin_amdgcn_raw_buffer_load_b128(res_c, (int)code_off, 0, 0);
    uint32_t sb_src = __builtin_amdgcn_raw_buffer_load_b8(res_s, (int)scale_off, 0, 0);
    uint32_t sw0 = 0u, sw1 = 0u;   // the row's scale bytes as the two dwords of the output's scale tile (groups h, 2+h, 4+h, 6+h)
    uint8_t* crow = codes + (size_t)out_row * (k >> 1) + (size_t)grp0 * 16u;   // the row's 128 bytes of codes in this K-quad
// One step g: fetch the next step's codes and scale byte (past the eighth step the values are not
// used), decode this step's, pass them through the wave's stage, quantize column `lane`.
#define REQUANT_STEP(G, OUT)                                                                            \
    {                                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        v4u_t cw_next = cw;                                                                             \
        uint32_t sb_next = sb_src;                                                                      \
        if ((G) + 1u < 8u) {                                                                            \
            cw_next = __builtin_amdgcn_raw_buffer_load_b128(res_c, (int)code_off, (int)(((G) + 1u) * code_step), 0); \
            sb_next = __builtin_amdgcn_raw_buffer_load_b8(res_s, (int)scale_off, (int)(((G) + 1u) * scale_step), 0); \
        }                                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        asm volatile("" : "+v"(sb_src)); /* the scale is formed here, not next to its load: no early wait */ \
        const float sc = u2f(sb_src << 23);                                                             \
        /* the sign vector applied on the codes: all 32 values of this lane are element rl of their groups */ \
        const uint32_t w[4] = {cw.x ^ code_flip, cw.y ^ code_flip, cw.z ^ code_flip, cw.w ^ code_flip}; \
        float f[32];                                                                                    \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
            v2f a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sc, 0);                              \
            v2f b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sc, 1);                              \
            v2f c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sc, 2);                              \
            v2f d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sc, 3);                              \
            f[8 * i] = a[0]; f[8 * i + 1] = a[1]; f[8 * i + 2] = b[0]; f[8 * i + 3] = b[1];             \
            f[8 * i + 4] = c[0]; f[8 * i + 5] = c[1]; f[8 * i + 6] = d[0]; f[8 * i + 7] = d[1];         \
        }                                                                                               \
        cw = cw_next;                                                                                   \
        sb_src = sb_next;                                                                               \
        /* The stage belongs to this wave alone and a wave's LDS operations complete in order, so the   \
           exchange needs no barrier and no fence (a fence would also wait for the loads just issued):  \
           only the compiler must keep the writes and the reads in program order. */                    \
        __builtin_amdgcn_wave_barrier();                                                                \
        _Pragma("unroll") for (uint32_t j = 0; j < 32; ++j) stage[(32u * ch + j) * kStageStride + wr] = f[j]; \
        __builtin_amdgcn_wave_barrier();                                                                \
        float v[32];                                                                                    \
        _Pragma("unroll") for (uint32_t q = 0; q < 8; ++q) {                                            \
            const float4 x = *reinterpret_cast<const float4*>(&stage[lane * kStageStride + ((4u * q + rot) & 31u)]); \
            v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;                 \
        }                                                                                               \
        uint32_t sb, mw;                                                                                \
        quantize_group<MODE, true>(v, p, ((uint64_t)out_row * k + (grp0 + (G)) * 32u) >> 4, OUT, sb, mw); \
        if ((G) & 1u) sw1 |= sb << (8u * ((G) >> 1));                                                   \
        else sw0 |= sb << (8u * ((G) >> 1));                                                            \
    }
    if (MODE == kBwdSr) {
        // Unrolled, with the instruction scheduler fenced at the step boundaries: each step's codes get
        // registers of their own, so the wait before decoding them lets the next step's loads stay in
        // flight; the row's 128 bytes of codes leave together at the end (a store inside the loop makes
        // every step wait for it before its registers can be reused).
        uint4 out[8];
#pragma unroll
        for (uint32_t g = 0; g < 8; ++g) REQUANT_STEP(g, out[g])
        __builtin_amdgcn_sched_barrier(0);
        if (out_row >= rows) return;
#pragma unroll
        for (uint32_t g = 0; g < 8; ++g)
            if (grp0 + g < gk) *reinterpret_cast<uint4*>(crow + 16u * g) = out[g];
    } else {
        // round-to-nearest: the unrolled form costs this variant more registers than a CU can give four
        // waves; it keeps the loop, and each step stores its own 16 bytes
#pragma unroll 1
        for (uint32_t g = 0; g < 8; ++g) {
            uint4 out;
            REQUANT_STEP(g, out)
            if (out_row < rows && grp0 + g < gk) *reinterpret_cast<uint4*>(crow + 16u * g) = out;
        }
        if (out_row >= rows) return;
    }
#undef REQUANT_STEP
    // scales: dwords (row, h = 0) and (row, h = 1) of the output's scale tile; a wave's 64 rows fill two
    // 128-byte runs per h
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
        const uint32_t w = h ? sw1 : sw0;
        if (grp0 + h >= gk) continue;
        uint32_t* dst = reinterpret_cast<uint32_t*>(scales + scale_tile_offset(out_row, grp0 + h, okq));
        if (grp0 + 6u + h < gk) {
            *dst = w;
        } else {
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (grp0 + 2u * q + h < gk) reinterpret_cast<uint8_t*>(dst)[q] = (uint8_t)(w >> (8u * q));
        }
    }
}

template <int MODE, int WPB>
__global__ void __launch_bounds__(64 * WPB, 4)   // 4 waves per SIMD: at most 128 registers
requant_transposed_kernel(const uint8_t* __restrict__ src_codes, const uint8_t* __restrict__ src_scales,
                          uint32_t rows, uint32_t k, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                          SrParams p) {
    __shared__ float s_stage[WPB][64 * kStageStride];
    // its place in a 256-column stretch, and the stretch
    uint32_t wave, quad;
    if (WPB == 1) {
        // One-wave blocks go to the 8 XCDs in turn.  The four waves of a stretch read the same 128-byte lines, so they
        // are the blocks b, b+8, b+16, b+24 of a run of 32: same XCD, one L2 fetch per line instead of four.  The grid
        // is padded to whole runs; the blocks past the last stretch leave at once.
        quad = (blockIdx.x >> 5) * 8u + (blockIdx.x & 7u);
        wave = (blockIdx.x >> 3) & 3u;
        if (quad * 256u >= rows) return;
    } else {
        const uint32_t gwave = blockIdx.x * (uint32_t)WPB + (threadIdx.x >> 6);   // wave of the whole launch along the columns
        wave = gwave & 3u;
        quad = gwave >> 2;
    }
    requant_transposed_wave<MODE>(src_codes, src_scales, rows, k, codes, scales, p, wave, quad, blockIdx.y, s_stage[threadIdx.x >> 6]);
}

// ------------------------------------------------------------------ the backward pass's three operand conversions in one launch
// dy^T quantized along the tokens (quant_transposed_tile), X_q and W_q re-quantized along their other dimension
// (requant_transposed_wave, four waves = one 256-column stretch per block): Algorithm 1 Backward needs all three before the
// two gradient products and none depends on another.  Launched one after the other, the re-quantizers leave most of the
// chip idle on weight-sized tensors and every kernel pays its own ramp-up and drain.  In one grid the re-quantizer blocks
// come first (W_q's, then X_q's) and the dy^T tiles fill the CUs as those finish.  (Spreading the re-quantizer blocks
// evenly among the tiles was measured slower than launching the kernels one by one: it breaks up the order in which
// neighbouring tiles write their lines.)
struct BwdOperandsMap {
    uint32_t n_rq_w, n_rq;           // re-quantizer blocks of W_q, and of W_q and X_q together: block indices [0, n_rq)
    uint32_t t_gx, w_quads, x_quads; // dy^T tiles per column tile row (K-quads); 256-column stretches of W_q^T, X_q^T
    FastDiv div_t_gx, div_w_quads, div_x_quads;
    uint32_t n_tiles_end;            // blocks [n_rq, n_tiles_end): dy^T tiles; blocks from n_tiles_end on: row tiles of dy (optional)
    uint32_t r_k_blocks;             // row tiles per 8 rows of dy
    FastDiv div_r_k_blocks;
};

template <int MODE>
__global__ void __launch_bounds__(256, 4)   // 128 registers: four blocks per CU (their LDS, 4 x 36 KB, fits too)
bwd_operands_kernel(const uint16_t* __restrict__ dy, uint32_t t_rows, uint32_t t_k, int64_t t_ldx,
                    uint8_t* __restrict__ t_codes, uint8_t* __restrict__ t_scales, SrParams t_p,
                    const uint8_t* __restrict__ x_src_codes, const uint8_t* __restrict__ x_src_scales, uint32_t x_rows, uint32_t x_k,
                    uint8_t* __restrict__ x_codes, uint8_t* __restrict__ x_scales, SrParams x_p,
                    const uint8_t* __restrict__ w_src_codes, const uint8_t* __restrict__ w_src_scales, uint32_t w_rows, uint32_t w_k,
                    uint8_t* __restrict__ w_codes, uint8_t* __restrict__ w_scales, SrParams w_p,
                    uint4* __restrict__ r_codes, uint8_t* __restrict__ r_scales, SrParams r_p, BwdOperandsMap map) {
    __shared__ __align__(16) uint8_t smem[4u * 64u * kStageStride * sizeof(float)];   // 36 KB: four re-quantizer stages
    static_assert(sizeof(smem) >= 128 * 8 * (16 + 1 + 4), "the dy^T tile's staging must fit as well");
    static_assert(sizeof(smem) >= 4 * 256 * 16 + 64 * 4, "the row tile's staging must fit as well");
    const uint32_t b = blockIdx.x;
    if (b < map.n_rq) {
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        float* stage = reinterpret_cast<float*>(smem) + wave * (64u * kStageStride);
        if (b < map.n_rq_w) {
            const uint32_t kq = fast_div(b, map.div_w_quads), quad = b - kq * map.w_quads;
            requant_transposed_wave<MODE>(w_src_codes, w_src_scales, w_rows, w_k, w_codes, w_scales, w_p, wave, quad, kq, stage);
        } else {
            const uint32_t j = b - map.n_rq_w;
            const uint32_t kq = fast_div(j, map.div_x_quads), quad = j - kq * map.x_quads;
            requant_transposed_wave<MODE>(x_src_codes, x_src_scales, x_rows, x_k, x_codes, x_scales, x_p, wave, quad, kq, stage);
        }
    } else if (b >= map.n_tiles_end) {
        // Q(dy) in row mode (the first operand of the dx product), for callers that want all four conversions in one launch:
        // dy is [t_k x t_rows] row-major, groups along its rows
        uint4 (*stage)[256] = reinterpret_cast<uint4 (*)[256]>(smem);
        uint32_t* s_scale = reinterpret_cast<uint32_t*>(smem + 4 * 256 * 16);
        quant_row_tile<MODE, false, false>(dy, t_k, t_rows >> 5, t_ldx, r_codes, r_scales, nullptr, r_p, map.r_k_blocks,
                                           map.div_r_k_blocks, b - map.n_tiles_end, stage, s_scale);
    } else {
        const uint32_t tb = b - map.n_rq;
        const uint32_t by = fast_div(tb, map.div_t_gx), bx = tb - by * map.t_gx;
        uint4* s_codes = reinterpret_cast<uint4*>(smem);
        uint32_t* s_mask = reinterpret_cast<uint32_t*>(smem + 128 * 8 * 16);
        uint8_t* s_scales = smem + 128 * 8 * 20;
        quant_transposed_tile<MODE, false>(dy, t_rows, t_k, t_ldx, t_codes, t_scales, nullptr, t_p, bx,
                                           transposed_column_tile(bx, by, (t_rows + 127u) >> 7), s_codes, s_scales, s_mask);
    }
}

// Re-quantization for Hadamard blocks of NB = 2, 4 or 8 groups (same tile, same stage).  The groups of
// a block are whole groups of source rows, so the group-combining stages come first, on the decoded
// values: for output group G (place j in its block) a lane decodes its 32 columns of the NB source
// rows (block group jj, row rl), eight values at a time, flips their signs and folds them through the
// butterfly tree down to place j; the 32-point stages follow after the transposition as usual.
template <int MODE, int NB>
__global__ void __launch_bounds__(256)
requant_transposed_block_kernel(const uint8_t* __restrict__ src_codes, const uint8_t* __restrict__ src_scales,
                                uint32_t rows, uint32_t k, uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                SrParams p) {
    __shared__ float s_stage[4][64 * kStageStride];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    float* stage = s_stage[wave];
    const uint32_t gk = k >> 5, okq = (k + 255u) >> 8;
    const uint32_t half = rows >> 1, skq = (rows + 255u) >> 8;
    const uint32_t c0 = blockIdx.x * 256u + wave * 64u, kq = blockIdx.y, grp0 = kq * 8u;
    const uint32_t rl = lane >> 1, ch = lane & 1u, cg = wave * 2u + ch;
    const uint32_t cb0 = blockIdx.x * 256u;
    const uint32_t src_rows = (k - grp0 * 32u) < 256u ? (k - grp0 * 32u) : 256u;
    const uint32_t src_cols = (rows - cb0) < 256u ? (rows - cb0) : 256u;
    const __amdgpu_buffer_rsrc_t res_c = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(src_codes + (size_t)grp0 * 32u * half + (cb0 >> 1)), 0,
        (int)((src_rows - 1u) * half + (src_cols >> 1)), 0x00020000);
    const size_t tile0 = ((size_t)grp0 * skq + (cb0 >> 8)) * 256u;
    const __amdgpu_buffer_rsrc_t res_s = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t*>(src_scales + tile0), 0, (int)((size_t)gk * skq * 256u - tile0), 0x00020000);
    const uint32_t code_off = rl * half + ((wave * 64u + 32u * ch) >> 1);
    const uint32_t scale_off = (((cg & 1u) << 5) + rl) * 4u + (cg >> 1);
    const uint32_t code_step = 32u * half, scale_step = skq * 256u;
    const uint32_t wr = (rl + 16u * ch) & 31u;
    const uint32_t out_row = c0 + lane, rot = (16u * (lane >> 5)) & 31u;
    const float norm = block_norm((uint32_t)NB);
    uint32_t sw0 = 0u, sw1 = 0u;
    uint8_t* crow = codes + (size_t)out_row * (k >> 1) + (size_t)grp0 * 16u;
#pragma unroll 1
    for (uint32_t g = 0; g < 8; ++g) {
        const uint32_t jb = g & ~((uint32_t)NB - 1u), j = g - jb;
        const uint32_t neg1 = (j & 1u) << 31, neg2 = (j & 2u) << 30, neg4 = (j & 4u) << 29;
        v4u_t cw[NB];
        float sc[NB];
        uint32_t flip[NB];
#pragma unroll
        for (uint32_t jj = 0; jj < (uint32_t)NB; ++jj) {
            cw[jj] = __builtin_amdgcn_raw_buffer_load_b128(res_c, (int)code_off, (int)((jb + jj) * code_step), 0);
            const uint32_t sbyte = __builtin_amdgcn_raw_buffer_load_b8(res_s, (int)scale_off, (int)((jb + jj) * scale_step), 0);
            sc[jj] = u2f(sbyte << 23);
            // the loads of a whole block may stay in registers across the steps that share it, the decoded values may
            // not (NB x 32 floats): a scale the compiler cannot see through keeps the decoding inside the step
            asm volatile("" : "+v"(sc[jj]));
            flip[jj] = ((p.sign_words[jj] >> rl) & 1u) << 31;   // element rl of block group jj
        }
        float f[32];
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            __builtin_amdgcn_sched_barrier(0);               // one dword of codes per group at a time
            float x[NB][8];
#pragma unroll
            for (uint32_t jj = 0; jj < (uint32_t)NB; ++jj) {
                const uint32_t w = cw[jj][q];
                v2f a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, sc[jj], 0);
                v2f b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, sc[jj], 1);
                v2f c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, sc[jj], 2);
                v2f d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, sc[jj], 3);
                const float t[8] = {a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
#pragma unroll
                for (uint32_t e = 0; e < 8; ++e) x[jj][e] = u2f(f2u(t[e]) ^ flip[jj]);
            }
#pragma unroll
            for (uint32_t e = 0; e < 8; ++e) {
                float y[NB / 2];
#pragma unroll
                for (uint32_t m = 0; m < (uint32_t)NB / 2u; ++m) y[m] = x[2 * m][e] + u2f(f2u(x[2 * m + 1][e]) ^ neg1);
                if (NB >= 4) {
#pragma unroll
                    for (uint32_t m = 0; m < (uint32_t)NB / 4u; ++m) y[m] = y[2 * m] + u2f(f2u(y[2 * m + 1]) ^ neg2);
                }
                if (NB >= 8) y[0] = y[0] + u2f(f2u(y[1]) ^ neg4);
                f[8 * q + e] = y[0];
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (uint32_t jx = 0; jx < 32; ++jx) stage[(32u * ch + jx) * kStageStride + wr] = f[jx];
        __builtin_amdgcn_wave_barrier();
        float v[32];
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            const float4 xx = *reinterpret_cast<const float4*>(&stage[lane * kStageStride + ((4u * q + rot) & 31u)]);
            v[4 * q] = xx.x; v[4 * q + 1] = xx.y; v[4 * q + 2] = xx.z; v[4 * q + 3] = xx.w;
        }
        __builtin_amdgcn_wave_barrier();
        fwht32_unscaled(v);
#pragma unroll
        for (int i = 0; i < 32; ++i) v[i] = v[i] * norm;
        uint4 out;
        uint32_t sb, mw;
        encode_group<MODE>(v, p, ((uint64_t)out_row * k + (grp0 + g) * 32u) >> 4, out, sb, mw);
        if (g & 1u) sw1 |= sb << (8u * (g >> 1));
        else sw0 |= sb << (8u * (g >> 1));
        if (out_row < rows && grp0 + g < gk) *reinterpret_cast<uint4*>(crow + 16u * g) = out;
    }
    if (out_row >= rows) return;
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
        const uint32_t w = h ? sw1 : sw0;
        if (grp0 + h >= gk) continue;
        uint32_t* dst = reinterpret_cast<uint32_t*>(scales + scale_tile_offset(out_row, grp0 + h, okq));
        if (grp0 + 6u + h < gk) {
            *dst = w;
        } else {
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (grp0 + 2u * q + h < gk) reinterpret_cast<uint8_t*>(dst)[q] = (uint8_t)(w >> (8u * q));
        }
    }
}

// ------------------------------------------------------------------ MXFP4 -> fp32
__global__ void __launch_bounds__(256)
dequant_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales, uint32_t n_groups,
               uint32_t gk, FastDiv div_gk, float* __restrict__ out) {
    uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g >= n_groups) return;
    uint4 q = reinterpret_cast<const uint4*>(codes)[g];
    const uint32_t row = fast_div(g, div_gk), gi = g - row * gk;
    float s = u2f((uint32_t)scales[scale_tile_offset(row, gi, (gk + 7u) >> 3)] << 23);
    uint32_t w[4] = {q.x, q.y, q.z, q.w};
    float4* dst = reinterpret_cast<float4*>(out + (size_t)g * 32u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v2f a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], s, 0);
        v2f b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], s, 1);
        v2f c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], s, 2);
        v2f d = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], s, 3);
        dst[2 * i] = make_float4(a[0], a[1], b[0], b[1]);
        dst[2 * i + 1] = make_float4(c[0], c[1], d[0], d[1]);
    }
}

// ------------------------------------------------------------------ host-side launchers

static FastDiv make_fast_div(uint32_t d) {
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    uint64_t mul = ((((uint64_t)1 << l) - d) << 32) / d + 1;
    return FastDiv{(uint32_t)mul, l};
}

template <int MODE, bool MASK>
static void launch_row_big(bool big, dim3 grid, hipStream_t st, const void* x, int64_t rows, uint32_t gk, int64_t ldx,
                           uint8_t* codes, uint8_t* scales, uint32_t* mask, const SrParams& p, uint32_t k_blocks) {
    dim3 block(256);
    if (big)
        hipLaunchKernelGGL((quant_row_kernel<MODE, MASK, true>), grid, block, 0, st, (const uint16_t*)x, (uint32_t)rows,
                           gk, ldx, (uint4*)codes, scales, mask, p, k_blocks, make_fast_div(k_blocks));
    else
        hipLaunchKernelGGL((quant_row_kernel<MODE, MASK, false>), grid, block, 0, st, (const uint16_t*)x, (uint32_t)rows,
                           gk, ldx, (uint4*)codes, scales, mask, p, k_blocks, make_fast_div(k_blocks));
}

template <int MODE>
static hipError_t launch_row(const void* x, int64_t rows, int64_t k, int64_t ldx, uint8_t* codes,
                             uint8_t* scales, uint32_t* mask, const SrParams& p, hipStream_t st) {
    if (rows == 0 || k == 0) return hipSuccess;
    const uint32_t gk = (uint32_t)(k / 32);
    const uint32_t k_blocks = (gk + 31) / 32;
    dim3 grid((uint32_t)((rows + 7) / 8) * k_blocks);
    if (mask) launch_row_big<MODE, true>(p.nb > 1u, grid, st, x, rows, gk, ldx, codes, scales, mask, p, k_blocks);
    else launch_row_big<MODE, false>(p.nb > 1u, grid, st, x, rows, gk, ldx, codes, scales, mask, p, k_blocks);
    return hipGetLastError();
}

template <int MODE, bool MASK>
static void launch_transposed_nb(dim3 grid, hipStream_t st, const void* src, int64_t rows, int64_t k, int64_t ldx,
                                 uint8_t* codes, uint8_t* scales, uint32_t* mask, const SrParams& p) {
    dim3 block(256);
    const uint16_t* s = (const uint16_t*)src;
    switch (p.nb) {
    case 1u: hipLaunchKernelGGL((quant_transposed_kernel<MODE, MASK>), grid, block, 0, st, s, (uint32_t)rows, (uint32_t)k, ldx, codes, scales, mask, p); break;
    case 2u: hipLaunchKernelGGL((quant_transposed_block_kernel<MODE, MASK, 2>), grid, block, 0, st, s, (uint32_t)rows, (uint32_t)k, ldx, codes, scales, mask, p); break;
    case 4u: hipLaunchKernelGGL((quant_transposed_block_kernel<MODE, MASK, 4>), grid, block, 0, st, s, (uint32_t)rows, (uint32_t)k, ldx, codes, scales, mask, p); break;
    default: hipLaunchKernelGGL((quant_transposed_block_kernel<MODE, MASK, 8>), grid, block, 0, st, s, (uint32_t)rows, (uint32_t)k, ldx, codes, scales, mask, p); break;
    }
}

template <int MODE>
static hipError_t launch_transposed(const void* src, int64_t rows, int64_t k, int64_t ldx, uint8_t* codes,
                                    uint8_t* scales, uint32_t* mask, const SrParams& p, hipStream_t st) {
    if (rows == 0 || k == 0) return hipSuccess;
    dim3 grid((uint32_t)((k / 32 + 7) / 8), (uint32_t)((rows + 127) / 128));
    if (mask) launch_transposed_nb<MODE, true>(grid, st, src, rows, k, ldx, codes, scales, mask, p);
    else launch_transposed_nb<MODE, false>(grid, st, src, rows, k, ldx, codes, scales, mask, p);
    return hipGetLastError();
}

hipError_t launch_quant(int mode, const void* x, int64_t rows, int64_t k, int64_t ldx, int transpose,
                        const SrParams& p, uint8_t* codes, uint8_t* scales, uint32_t* mask, hipStream_t st) {
    if (!transpose) {
        switch (mode) {
        case kFwd: return launch_row<kFwd>(x, rows, k, ldx, codes, scales, mask, p, st);
        case kBwdRtn: return launch_row<kBwdRtn>(x, rows, k, ldx, codes, scales, nullptr, p, st);
        default: return launch_row<kBwdSr>(x, rows, k, ldx, codes, scales, nullptr, p, st);
        }
    }
    switch (mode) {
    case kFwd: return launch_transposed<kFwd>(x, rows, k, ldx, codes, scales, mask, p, st);
    case kBwdRtn: return launch_transposed<kBwdRtn>(x, rows, k, ldx, codes, scales, nullptr, p, st);
    default: return launch_transposed<kBwdSr>(x, rows, k, ldx, codes, scales, nullptr, p, st);
    }
}

template <int MODE>
static void launch_requant_nb(dim3 grid, hipStream_t st, const uint8_t* src_codes, const uint8_t* src_scales, int64_t rows,
                              int64_t k, const SrParams& p, uint8_t* codes, uint8_t* scales) {
    dim3 block(256);
    switch (p.nb) {
    case 1u:
        // one wave per block (the waves never cooperate): measured equal to four-wave blocks on the large tensors and
        // 8-20 % faster on weight-sized ones, where it spreads the same waves over four times as many CUs; runs of 32
        // blocks = 8 stretches x 4 waves, see the kernel
        hipLaunchKernelGGL((requant_transposed_kernel<MODE, 1>), dim3(((grid.x + 7u) / 8u) * 32u, grid.y), dim3(64), 0, st, src_codes, src_scales, (uint32_t)rows, (uint32_t)k, codes, scales, p);
        break;
    case 2u: hipLaunchKernelGGL((requant_transposed_block_kernel<MODE, 2>), grid, block, 0, st, src_codes, src_scales, (uint32_t)rows, (uint32_t)k, codes, scales, p); break;
    case 4u: hipLaunchKernelGGL((requant_transposed_block_kernel<MODE, 4>), grid, block, 0, st, src_codes, src_scales, (uint32_t)rows, (uint32_t)k, codes, scales, p); break;
    default: hipLaunchKernelGGL((requant_transposed_block_kernel<MODE, 8>), grid, block, 0, st, src_codes, src_scales, (uint32_t)rows, (uint32_t)k, codes, scales, p); break;
    }
}

hipError_t launch_requant_transpose(int mode, const uint8_t* src_codes, const uint8_t* src_scales,
                                    int64_t rows, int64_t k, const SrParams& p, uint8_t* codes,
                                    uint8_t* scales, hipStream_t st) {
    if (rows == 0 || k == 0) return hipSuccess;
    dim3 grid((uint32_t)((rows + 255) / 256), (uint32_t)((k + 255) / 256));
    if (mode == kBwdRtn) launch_requant_nb<kBwdRtn>(grid, st, src_codes, src_scales, rows, k, p, codes, scales);
    else launch_requant_nb<kBwdSr>(grid, st, src_codes, src_scales, rows, k, p, codes, scales);
    return hipGetLastError();
}

hipError_t launch_fwd_operands(const void* x, int64_t tokens, const void* w, int64_t out, int64_t in, uint8_t* xq_codes,
                               uint8_t* xq_scales, uint32_t* x_mask, uint8_t* wq_codes, uint8_t* wq_scales, uint32_t* w_mask,
                               const SrParams& p, hipStream_t st) {
    if (in == 0 || (tokens == 0 && out == 0)) return hipSuccess;
    const uint32_t gk = (uint32_t)(in / 32);
    const uint32_t k_blocks = (gk + 31) / 32;
    const uint64_t na = (uint64_t)((tokens + 7) / 8) * k_blocks, nb = (uint64_t)((out + 7) / 8) * k_blocks;
    if (na + nb >= ((uint64_t)1 << 31)) return hipErrorInvalidValue;
    RowMatrix a = {(const uint16_t*)x, (uint32_t)tokens, in, (uint4*)xq_codes, xq_scales, x_mask};
    RowMatrix b = {(const uint16_t*)w, (uint32_t)out, in, (uint4*)wq_codes, wq_scales, w_mask};
    hipLaunchKernelGGL((quant_row_pair_kernel<kFwd, true>), dim3((uint32_t)(na + nb)), dim3(256), 0, st, a, b, (uint32_t)na, gk, p,
                       k_blocks, make_fast_div(k_blocks));
    return hipGetLastError();
}

hipError_t launch_bwd_operands(int mode, const void* dy, int64_t tokens, int64_t in, int64_t out,
                               const uint8_t* xq_codes, const uint8_t* xq_scales, const uint8_t* wq_codes, const uint8_t* wq_scales,
                               const SrParams& p_dyt, const SrParams& p_x, const SrParams& p_w,
                               uint8_t* dyt_codes, uint8_t* dyt_scales, uint8_t* xt_codes, uint8_t* xt_scales,
                               uint8_t* wt_codes, uint8_t* wt_scales,
                               const SrParams& p_dy, uint8_t* dy_codes, uint8_t* dy_scales, hipStream_t st) {
    BwdOperandsMap map;
    // dy^T: logical [out x tokens]; X_q^T: [in x tokens] from [tokens x in]; W_q^T: [in x out] from [out x in].
    // An empty dimension empties the conversions it belongs to, not the others.
    map.t_gx = (uint32_t)((tokens / 32 + 7) / 8);
    const uint32_t t_gy = (uint32_t)((out + 127) / 128);
    map.w_quads = map.x_quads = (uint32_t)((in + 255) / 256);
    map.n_rq_w = map.w_quads * (uint32_t)((out + 255) / 256);
    map.n_rq = map.n_rq_w + map.x_quads * (uint32_t)((tokens + 255) / 256);
    uint64_t total = (uint64_t)map.t_gx * t_gy + map.n_rq;
    if (total >= ((uint64_t)1 << 31)) return hipErrorInvalidValue;
    map.n_tiles_end = (uint32_t)total;
    // optional fourth conversion: dy [tokens x out] in row mode, 8 rows x 1024 columns per block
    map.r_k_blocks = (uint32_t)((out / 32 + 31) / 32);
    if (dy_codes) total += (uint64_t)((tokens + 7) / 8) * map.r_k_blocks;
    if (total == 0) return hipSuccess;
    if (total >= ((uint64_t)1 << 31)) return hipErrorInvalidValue;
    map.div_t_gx = make_fast_div(map.t_gx ? map.t_gx : 1u);
    map.div_w_quads = make_fast_div(map.w_quads ? map.w_quads : 1u);
    map.div_x_quads = make_fast_div(map.x_quads ? map.x_quads : 1u);
    map.div_r_k_blocks = make_fast_div(map.r_k_blocks ? map.r_k_blocks : 1u);
    dim3 grid((uint32_t)total), block(256);
    if (mode == kBwdRtn)
        hipLaunchKernelGGL((bwd_operands_kernel<kBwdRtn>), grid, block, 0, st, (const uint16_t*)dy, (uint32_t)out, (uint32_t)tokens, out,
                           dyt_codes, dyt_scales, p_dyt, xq_codes, xq_scales, (uint32_t)in, (uint32_t)tokens, xt_codes, xt_scales, p_x,
                           wq_codes, wq_scales, (uint32_t)in, (uint32_t)out, wt_codes, wt_scales, p_w,
                           reinterpret_cast<uint4*>(dy_codes), dy_scales, p_dy, map);
    else
        hipLaunchKernelGGL((bwd_operands_kernel<kBwdSr>), grid, block, 0, st, (const uint16_t*)dy, (uint32_t)out, (uint32_t)tokens, out,
                           dyt_codes, dyt_scales, p_dyt, xq_codes, xq_scales, (uint32_t)in, (uint32_t)tokens, xt_codes, xt_scales, p_x,
                           wq_codes, wq_scales, (uint32_t)in, (uint32_t)out, wt_codes, wt_scales, p_w,
                           reinterpret_cast<uint4*>(dy_codes), dy_scales, p_dy, map);
    return hipGetLastError();
}

hipError_t launch_dequant(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t k, float* out,
                          hipStream_t st) {
    uint64_t n_groups = (uint64_t)rows * (uint64_t)(k / 32);
    if (n_groups == 0) return hipSuccess;
    dim3 grid((uint32_t)((n_groups + 255) / 256)), block(256);
    hipLaunchKernelGGL(dequant_kernel, grid, block, 0, st, codes, scales, (uint32_t)n_groups, (uint32_t)(k / 32),
                       make_fast_div((uint32_t)(k / 32)), out);
    return hipGetLastError();
}

}  // namespace quartet
