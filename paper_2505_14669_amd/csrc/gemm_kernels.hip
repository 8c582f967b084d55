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
// Kernels: gemm_mxfp4_stream_kernel (256 x 256 tiles) and gemm_mxfp4_stream_tile_kernel (128 x 256 and 128 x 128 tiles
// for small problems): one block per compute unit streams its tiles through a ring of LDS stages.  Both work
// through a batch of one or two products per launch (GemmBatch).
#include "gemm_common.h"
#include "launchers.h"

namespace quartet {

// Test / tuning override of the kernel choice (quartet_debug_set_gemm_plan): -1 / 0 = the size heuristics below.
static int g_forced_variant = -1;
static int g_forced_band = 0;

// quartet_profile_clock: device counters the streaming kernel adds each block's run time to (null: off)
static uint64_t* g_clock_counters = nullptr;

void set_clock_counters(uint64_t* device_counters) { g_clock_counters = device_counters; }

void set_gemm_plan(int variant, int band_height) {
    g_forced_variant = variant;
    g_forced_band = band_height;
}

// One product of a launch of the 256 x 256 streaming kernel, and the one or two products a launch works through: the
// block's virtual tile ids run over the first product's tiles, then the second's (Algorithm 1 Backward: the two gradient
// products do not depend on each other; in one launch the second starts where the first leaves compute units idle and
// there is one ramp-up and one drain instead of two).
struct GemmProblem {
    const uint8_t* a_codes;
    const uint8_t* a_scales;
    const uint8_t* b_codes;
    const uint8_t* b_scales;
    void* d;
    const uint32_t* mask;
    uint32_t m, n, k, ldd;
    float alpha;
    uint32_t tiles_m, tiles_n, band_height, total_tiles;
};
struct GemmBatch {
    GemmProblem p[2];
};

template <int S>
__device__ __forceinline__ v16f mfma_fp4(const uint4& a, const uint4& b, v16f c, uint32_t sa, uint32_t sb) {
    v8i va = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    v8i vb = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, c, 4, 4, S, (int)sa, S, (int)sb);
}

// ---------------------------------------------------------------------------------------------
// Streaming variant: one block per compute unit walks its tiles (virtual block ids b, b + G, ...), and the ring of LDS
// stages never drains between them: the loads of the next tile's first stages are issued during the last stages
// of the current one, so a tile's first matrix-core instruction follows the previous tile's result stores directly.
// The epilogue uses a scratch of its own (16 KB beside the 144 KB ring).
template <bool OUT_BF16, bool FUSED>
__global__ void __launch_bounds__(256)
gemm_mxfp4_stream_kernel(GemmBatch batch, uint32_t total_tiles, uint32_t nb, uint64_t* __restrict__ clock_counters) {
    constexpr uint32_t TM = 4, TN = 4, BM = 256, BN = 256;
    constexpr uint32_t CODES = (BM + BN) * 4;            // 16-byte chunks of codes per stage
    constexpr uint32_t STAGE = CODES + 256;              // + 16 scale tiles of 256 B
    constexpr uint32_t D = kRing - 1;                    // prefetch distance in stages
    constexpr uint32_t EPI = 4u * 256u;                  // 16-byte chunks of epilogue scratch (4 KB per wave)
    __shared__ uint4 lds[kRing * STAGE + EPI];

    // measurement support: shader-clock and constant-clock ticks of this block's run (wave-uniform branch)
    uint64_t clk_t0 = 0, clk_w0 = 0;
    if (clock_counters) {
        clk_t0 = __builtin_readcyclecounter();
        clk_w0 = __builtin_amdgcn_s_memrealtime();
    }

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
    const uint32_t G = gridDim.x, first_tiles = batch.p[0].total_tiles;
    const uint32_t wm0 = (wave >> 1) * 128u, wn0 = (wave & 1u) * 128u;
    const bool scales_of_a = wave < 2u;

// product SEL and the tile's number in it for virtual block id V (ids past the last tile: a number past the product's tiles)
#define STREAM_PRODUCT(V, SEL, LOCAL)                                                                   \
    {                                                                                                   \
        LOCAL = (V);                                                                                    \
        SEL = 0u;                                                                                       \
        if (LOCAL >= first_tiles) { LOCAL -= first_tiles; SEL = 1u; }                                   \
    }
// tile origin of tile number V of product Q (XCD-aware order, bands of band_height tile rows); V >= its tiles: M0 = m (no rows)
#define STREAM_TILE(Q, V, M0, N0)                                                                       \
    {                                                                                                   \
        const uint32_t v_ = (V), tt_ = (Q).total_tiles;                                                 \
        if (v_ < tt_) {                                                                                 \
            const uint32_t per_ = tt_ >> 3, rem_ = tt_ & 7u, GM_ = (Q).band_height;                     \
            const uint32_t tiles_m_ = (Q).tiles_m, tiles_n_ = (Q).tiles_n;                              \
            const uint32_t xcd_ = v_ & 7u;                                                              \
            const uint32_t tile_ = xcd_ * per_ + (xcd_ < rem_ ? xcd_ : rem_) + (v_ >> 3);               \
            const uint32_t band_ = tile_ / (GM_ * tiles_n_);                                            \
            const uint32_t band_rows_ = (tiles_m_ - band_ * GM_) < GM_ ? (tiles_m_ - band_ * GM_) : GM_; \
            const uint32_t in_band_ = tile_ - band_ * GM_ * tiles_n_;                                   \
            M0 = (band_ * GM_ + in_band_ % band_rows_) * BM;                                            \
            N0 = (in_band_ / band_rows_) * BN;                                                          \
        } else {                                                                                        \
            M0 = (Q).m; N0 = (Q).n;                                                                     \
        }                                                                                               \
    }
    // issue cursor: the tile and stage the next LDS-direct loads belong to
    // (its product's inner dimension decides the offsets: kb = bytes per code row, kq = K-quads, S2i = stages per tile)
    // A tile does not start at K = 0: the tiles of XCD class c (tile number mod 8; an XCD's compute units hold tiles of
    // one class at a time and must stay in step to share panels in their L2) start c/8 of the way along K, in whole K-quads,
    // and wrap around: ikst is the K-stage the cursor's local stage ist stands for.  Otherwise every compute unit of the
    // chip asks for the same few hundred bytes of its operand rows at the same time, and with a row pitch of a few KB the
    // memory channels behind the L2s serve that unevenly (measured: 1-2 % of the K = 4096 products' time).  fp32 sums are
    // formed in a rotated order then, the same for a tile wherever it runs.  Only for K a multiple of 256: a ragged last
    // K-quad keeps its place at the end.
    uint32_t iv = blockIdx.x, ist = 0u;
    v4i_t res_a, res_b, res_s;
    uint32_t kb, istages, S2i, goff, gstep, soff, ikst;
    const uint32_t drow = wave * 16u + (lane >> 2);
    const uint32_t dcol = (lane & 3u) ^ ((drow >> 2) & 3u);
#define STREAM_ISSUE_SETUP()                                                                            \
    {                                                                                                   \
        uint32_t sel_, lv_, m0_, n0_;                                                                   \
        STREAM_PRODUCT(iv, sel_, lv_)                                                                   \
        const GemmProblem& q_ = batch.p[sel_];                                                          \
        STREAM_TILE(q_, lv_, m0_, n0_)                                                                  \
        const uint32_t k_ = q_.k, kq_ = (k_ + 255u) >> 8;                                               \
        kb = k_ >> 1;                                                                                   \
        istages = (k_ + 127u) >> 7;                                                                     \
        S2i = istages < 2u ? 2u : ((istages + 1u) & ~1u);                                               \
        ikst = ((k_ & 255u) == 0u) ? (((lv_ & 7u) * (S2i >> 1)) >> 3) * 2u : 0u;                        \
        goff = drow * kb + dcol * 16u;          /* + j*64*kb, + stage*64 */                             \
        gstep = 64u * kb;                                                                               \
        soff = (((wave & 1u) * 4u + (lane >> 4)) * kq_) * 256u + (lane & 15u) * 16u;   /* + quad*256 */ \
        const uint32_t rows_a_ = (q_.m - m0_) < BM ? (q_.m - m0_) : BM, rows_b_ = (q_.n - n0_) < BN ? (q_.n - n0_) : BN; \
        res_a = make_rsrc_words(q_.a_codes + (size_t)m0_ * kb, rows_a_ * kb);                           \
        res_b = make_rsrc_words(q_.b_codes + (size_t)n0_ * kb, rows_b_ * kb);                           \
        const uint32_t srow0_ = scales_of_a ? m0_ : n0_, srows_ = scales_of_a ? rows_a_ : rows_b_;      \
        res_s = make_rsrc_words((scales_of_a ? q_.a_scales : q_.b_scales) + (size_t)(srow0_ >> 5) * kq_ * 256u, \
                                ((srows_ + 31u) >> 5) * kq_ * 256u);                                    \
    }
    STREAM_ISSUE_SETUP()

    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)&lds[0];
    const uint32_t swz = (lrow >> 2) & 3u;
    const uint32_t fa_base = (wm0 + lrow) * 4u, fb_base = BM * 4u + (wn0 + lrow) * 4u;
    const uint32_t sa_base = CODES * 4u + (wm0 >> 5) * 64u + lane;             // dword index in a stage
    const uint32_t sb_base = CODES * 4u + 8u * 64u + (wn0 >> 5) * 64u + lane;

    uint32_t sa[TM], sb[TN], ra_n[TM], rb_n[TN];
    uint4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];

// load J (0..3: A rows, 4..7: B rows, 8: scale tiles) of the issue cursor's stage into ring slot SLOT
#define STREAM_ISSUE(SLOT, J)                                                                           \
    {                                                                                                   \
        const uint32_t slot_ = lds0 + ((SLOT) * STAGE + wave * 64u) * 16u;                              \
        if ((J) < 8u) {                                                                                 \
            const uint32_t base_ = (ikst * 64u + dcol * 16u < kb) ? goff + ikst * 64u : kOutOfRange;      \
            lds_direct_load16((J) < 4u ? res_a : res_b, base_ + ((J) & 3u) * gstep, slot_ + (J) * 4096u); \
        } else {                                                                                        \
            lds_direct_load16(res_s, (ikst < istages) ? soff + (ikst >> 1) * 256u : kOutOfRange, slot_ + CODES * 16u); \
        }                                                                                               \
    }
// the stage is issued: move the cursor on (to the next tile of this block after the tile's last stage)
#define STREAM_ISSUE_ADVANCE()                                                                          \
    {                                                                                                   \
        ++ist;                                                                                          \
        ++ikst;                                                                                         \
        if (ikst == S2i) ikst = 0u;                                                                     \
        if (ist == S2i) {                                                                               \
            ist = 0u;                                                                                   \
            iv += G;                                                                                    \
            STREAM_ISSUE_SETUP()                                                                        \
        }                                                                                               \
    }
#define STREAM_FRAG_A(SLOT, S, FA, I) FA[I] = lds[(SLOT) * STAGE + fa_base + (I) * 128u + ((2u * (S) + lhalf) ^ swz)];
#define STREAM_FRAG_B(SLOT, S, FB, J) FB[J] = lds[(SLOT) * STAGE + fb_base + (J) * 128u + ((2u * (S) + lhalf) ^ swz)];
#define STREAM_FENCE() __builtin_amdgcn_sched_barrier(0);

    constexpr uint32_t KEEP2 = 17u;                    // loads of one even and one odd stage stay in flight
    constexpr uint32_t WAIT2 = 0x0F70u | (KEEP2 & 15u) | ((KEEP2 >> 4) << 14);
#pragma unroll
    for (uint32_t s0 = 0; s0 < D; ++s0) {
#pragma unroll
        for (uint32_t j = 0; j < 8u; ++j) STREAM_ISSUE(s0, j)
        if ((s0 & 1u) == 0u) STREAM_ISSUE(s0, 8u)
        STREAM_ISSUE_ADVANCE()
    }
    __builtin_amdgcn_s_waitcnt(WAIT2);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (uint32_t i = 0; i < TM; ++i) { STREAM_FRAG_A(0u, 0u, fa0, i) STREAM_FRAG_B(0u, 0u, fb0, i) }
// Scale dwords of a K-quad, in two steps a few hundred cycles apart: the raw dwords are read from ring slot SLOT right
// behind the barrier that makes them visible, and turned into the operands of the next pair of stages (the K-quad that
// starts with the even local stage ST of a tile whose product has GK groups along K; bytes of groups past GK become 2^0)
// only behind the current pair's last matrix-core instruction.  Used at once, the reads made the wave wait for every LDS
// read in flight at the end of each odd stage.
#define STREAM_SCALES_READ(SLOT)                                                                        \
    {                                                                                                   \
        const uint32_t* sbuf_ = reinterpret_cast<const uint32_t*>(&lds[(SLOT) * STAGE]);                \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) ra_n[i] = sbuf_[sa_base + i * 64u];         \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) rb_n[j] = sbuf_[sb_base + j * 64u];         \
    }
#define STREAM_SCALES_USE(ST, GK)                                                                       \
    {                                                                                                   \
        uint32_t keep_ = 0xFFFFFFFFu;                                                                   \
        if (((ST) + 2u) * 4u > (GK)) {        /* wave-uniform: only a ragged last K-quad */             \
            const uint32_t ksteps_lane = ((GK) + 1u - lhalf) >> 1;   /* K-steps in which this half-wave has a group */ \
            const uint32_t done_ = (ST) * 2u;                                                           \
            const uint32_t nv_ = ksteps_lane > done_ ? (ksteps_lane - done_ < 4u ? ksteps_lane - done_ : 4u) : 0u; \
            keep_ = nv_ >= 4u ? 0xFFFFFFFFu : ((1u << (8u * nv_)) - 1u);                                \
        }                                                                                               \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) sa[i] = (ra_n[i] & keep_) | (0x7F7F7F7Fu & ~keep_); \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) sb[j] = (rb_n[j] & keep_) | (0x7F7F7F7Fu & ~keep_); \
    }
    uint32_t csel, clv;
    STREAM_PRODUCT(blockIdx.x, csel, clv)
    STREAM_SCALES_READ(0u)
    STREAM_SCALES_USE(0u, batch.p[csel].k >> 5)
#define STREAM_MF(S, FA, FB, I, J)                                                                      \
    acc[I][J] = mfma_fp4<S>(FA[I], FB[J], acc[I][J], sa[I], sb[J]);                                     \
    asm volatile("" : "+a"(acc[I][J]));                                                                 \
    STREAM_FENCE()
// one stage: PAR = its parity, ST = its local index, slots: SL = its own, SL1 = the next stage's, SLI = the one being filled
#define STREAM_BODY(PAR, ST, SL, SL1, SLI, NEXT_ST, NEXT_GK)                                            \
    {                                                                                                   \
        STREAM_MF(2 * PAR, fa0, fb0, 0, 0) STREAM_FRAG_B(SL, 1u, fb1, 0) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 0, 1) STREAM_FRAG_B(SL, 1u, fb1, 1) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 0, 2) STREAM_FRAG_B(SL, 1u, fb1, 2) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 0, 3) STREAM_FRAG_B(SL, 1u, fb1, 3) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 1, 0) STREAM_FRAG_A(SL, 1u, fa1, 0) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 1, 1) STREAM_FRAG_A(SL, 1u, fa1, 1) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 1, 2) STREAM_FRAG_A(SL, 1u, fa1, 2) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 1, 3) STREAM_FRAG_A(SL, 1u, fa1, 3) STREAM_FENCE()                 \
        STREAM_MF(2 * PAR, fa0, fb0, 2, 0) STREAM_ISSUE(SLI, 0u) STREAM_FENCE()                         \
        STREAM_MF(2 * PAR, fa0, fb0, 2, 1)                                                              \
        STREAM_MF(2 * PAR, fa0, fb0, 2, 2) STREAM_ISSUE(SLI, 1u) STREAM_FENCE()                         \
        STREAM_MF(2 * PAR, fa0, fb0, 2, 3)                                                              \
        STREAM_MF(2 * PAR, fa0, fb0, 3, 0) STREAM_ISSUE(SLI, 2u) STREAM_FENCE()                         \
        STREAM_MF(2 * PAR, fa0, fb0, 3, 1)                                                              \
        STREAM_MF(2 * PAR, fa0, fb0, 3, 2) STREAM_ISSUE(SLI, 3u) STREAM_FENCE()                         \
        STREAM_MF(2 * PAR, fa0, fb0, 3, 3)                                                              \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 0, 0) STREAM_ISSUE(SLI, 4u) STREAM_FENCE()                     \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 0, 1)                                                          \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 0, 2) STREAM_ISSUE(SLI, 5u) STREAM_FENCE()                     \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 0, 3)                                                          \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 1, 0) STREAM_ISSUE(SLI, 6u) STREAM_FENCE()                     \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 1, 1)                                                          \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 1, 2) STREAM_ISSUE(SLI, 7u) STREAM_FENCE()                     \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 1, 3)                                                          \
        if (PAR == 1) { STREAM_ISSUE(SLI, 8u) STREAM_FENCE() }   /* the stage being filled is even */   \
        STREAM_ISSUE_ADVANCE()                                                                          \
        __builtin_amdgcn_s_waitcnt(WAIT2);                                                              \
        __builtin_amdgcn_s_barrier();                                                                   \
        STREAM_FENCE()                                                                                  \
        if (PAR == 1) { STREAM_SCALES_READ(SL1) STREAM_FENCE() }                                        \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 2, 0) STREAM_FRAG_A(SL1, 0u, fa0, 0) STREAM_FRAG_B(SL1, 0u, fb0, 0) STREAM_FENCE() \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 2, 1) STREAM_FRAG_B(SL1, 0u, fb0, 1) STREAM_FRAG_B(SL1, 0u, fb0, 2) STREAM_FENCE() \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 2, 2) STREAM_FRAG_B(SL1, 0u, fb0, 3) STREAM_FENCE()            \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 2, 3) STREAM_FRAG_A(SL1, 0u, fa0, 1) STREAM_FENCE()            \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 3, 0) STREAM_FRAG_A(SL1, 0u, fa0, 2) STREAM_FENCE()            \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 3, 1) STREAM_FRAG_A(SL1, 0u, fa0, 3) STREAM_FENCE()            \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 3, 2)                                                          \
        STREAM_MF(2 * PAR + 1, fa1, fb1, 3, 3)                                                          \
        if (PAR == 1) { STREAM_SCALES_USE(NEXT_ST, NEXT_GK) STREAM_FENCE() }                            \
    }

    v16f acc[TM][TN];
    float* wbuf = reinterpret_cast<float*>(&lds[kRing * STAGE]) + wave * 1024u;
    uint32_t g = 0u;                                       // stages done by this block (ring slot = g % kRing)
    for (uint32_t cv = blockIdx.x; cv < total_tiles; cv += G) {
        STREAM_PRODUCT(cv, csel, clv)
        const uint32_t ck = batch.p[csel].k, gk = ck >> 5, stages = (ck + 127u) >> 7;
        const uint32_t S2 = stages < 2u ? 2u : ((stages + 1u) & ~1u);   // stages per tile, even (extra stages are zero-filled)
        // the tile's last pair of stages reads the first scales of the block's next tile, which may belong to the other product
        const uint32_t gk_after = (cv + G >= first_tiles && cv + G < total_tiles) ? (batch.p[1].k >> 5) : gk;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        for (uint32_t st = 0u; st < S2; st += 2u, g += 2u) {
            const uint32_t sl = g & 3u;                    // g is even: sl is 0 or 2
            const uint32_t next_st = st + 2u < S2 ? st + 2u : 0u;   // after the tile's last pair: the next tile's stage 0
            const uint32_t next_gk = st + 2u < S2 ? gk : gk_after;
            STREAM_BODY(0, st, sl, sl + 1u, sl ^ 3u, 0u, 0u)                    /* fills slot (g + 3) % 4 */
            STREAM_BODY(1, st + 1u, sl + 1u, sl ^ 2u, sl, next_st, next_gk)     /* fills slot (g + 4) % 4 */
        }
        // The ring already holds (or is receiving) the next tile's first stages, and fa0 / fb0 / sa / sb its first
        // fragments and scales.  The result stores below are older than every load issued from here on and the
        // vector-memory counter retires in order, so the next tile's first wait also waits for them.
        const GemmProblem& q = batch.p[csel];
        uint32_t m0, n0;
        STREAM_TILE(q, clv, m0, n0)
        const uint32_t m = q.m, n = q.n, ldd = q.ldd;
        const uint32_t* __restrict__ mask = q.mask;
        const uint32_t row_base = m0 + wm0, col_base = n0 + wn0;
        const bool full = (ldd & 3u) == 0u && row_base + TM * 32u <= m && col_base + TN * 32u <= n && (!FUSED || mask != nullptr);
        if (full) store_tile_rows8<TM, TN, OUT_BF16, FUSED, true>(acc, wbuf, q.d, ldd, mask, q.alpha, row_base, col_base, m, n, lane, nb);
        else store_tile_rows8<TM, TN, OUT_BF16, FUSED, false>(acc, wbuf, q.d, ldd, mask, q.alpha, row_base, col_base, m, n, lane, nb);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // the stages issued past the last tile (zero-filled) have landed before the LDS is given back
    if (clock_counters && tid == 0) {
        const uint64_t t1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
        atomicAdd(reinterpret_cast<unsigned long long*>(clock_counters), (unsigned long long)(t1 - clk_t0));
        atomicAdd(reinterpret_cast<unsigned long long*>(clock_counters) + 1, (unsigned long long)(w1 - clk_w0));
    }
#undef STREAM_PRODUCT
#undef STREAM_TILE
#undef STREAM_ISSUE_SETUP
#undef STREAM_ISSUE
#undef STREAM_ISSUE_ADVANCE
#undef STREAM_FRAG_A
#undef STREAM_FRAG_B
#undef STREAM_FENCE
#undef STREAM_SCALES_READ
#undef STREAM_SCALES_USE
#undef STREAM_MF
#undef STREAM_BODY
}

// ---------------------------------------------------------------------------------------------
// The streaming design for other tile shapes: wave tile (TM*32) x (TN*32), block tile (64 TM) x (64 TN), for problems
// whose 256 x 256 tiles would leave compute units idle.  Same ring, same issue cursor, same epilogue; the stage's
// instruction order is generated from the tile shape instead of written out: after matrix-core instruction number idx of
// a stage come, in this order, the fragment reads of the stage's second K-step (RPS per slot from slot 0), the stage's
// LDS-direct loads (spread over the slots up to the barrier), the wait and the barrier POST instructions before the
// stage's end, and behind the barrier the next stage's first fragments (and, on odd stages, the next K-quad's scales).
template <int TM, int TN, bool OUT_BF16, bool FUSED>
__global__ void __launch_bounds__(256)
gemm_mxfp4_stream_tile_kernel(GemmBatch batch, uint32_t total_tiles, uint32_t nb, uint64_t* __restrict__ clock_counters) {
    constexpr uint32_t BM = 64 * TM, BN = 64 * TN;
    static_assert(BM % 128 == 0 && BN % 128 == 0, "a wave's four scale tiles must belong to one operand");
    constexpr uint32_t CODES = (BM + BN) * 4;            // 16-byte chunks of codes per stage
    constexpr uint32_t STAGE = CODES + 256;              // + room for 16 scale tiles of 256 B (one KB per wave)
    constexpr uint32_t D = kRing - 1;
    constexpr uint32_t EPI = 4u * TN * 64u;              // 16-byte chunks of epilogue scratch: 8 rows x TN*32 floats per wave
    constexpr uint32_t LA = BM / 64, LB = BN / 64, NL = LA + LB;   // LDS-direct loads of codes per wave per stage
    constexpr uint32_t NT = (BM + BN) / 32;              // scale tiles per K-quad: A's, then B's
    constexpr int NM = TM * TN, R = TM + TN;             // matrix-core instructions and fragment reads per K-step
    constexpr int POST = NM >= 16 ? 8 : (NM >= 8 ? 6 : 3);   // matrix-core instructions behind the barrier
    constexpr int P = 2 * NM - POST;                     // slots in front of the barrier
    constexpr int RPS = (2 * R > NM) ? 2 : 1;            // second-K-step fragment reads per slot
    constexpr int RS_END = (R + RPS - 1) / RPS;          // first slot without such a read
    constexpr int XR = R - (POST > 2 ? POST - 2 : 1);    // reads of the next stage's first fragments that must double up
    static_assert(RS_END <= NM && RS_END < P, "the fragments of the second K-step must be read during the first");
    __shared__ uint4 lds[kRing * STAGE + EPI];

    // measurement support: shader-clock and constant-clock ticks of this block's run (wave-uniform branch)
    uint64_t clk_t0 = 0, clk_w0 = 0;
    if (clock_counters) {
        clk_t0 = __builtin_readcyclecounter();
        clk_w0 = __builtin_amdgcn_s_memrealtime();
    }

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
    const uint32_t G = gridDim.x, first_tiles = batch.p[0].total_tiles;
    const uint32_t wm0 = (wave >> 1) * (TM * 32u), wn0 = (wave & 1u) * (TN * 32u);
    // scale tiles 4 wave .. 4 wave + 3 of [A's | B's] are this wave's to fetch (waves past the last tile fetch nothing real:
    // their load is out of range and delivers zeros, which keeps every wave's count of loads the same)
    const bool has_scales = 4u * wave < NT, scales_of_a = 4u * wave < BM / 32u;
    const uint32_t stile0 = scales_of_a ? 4u * wave : 4u * wave - BM / 32u;

// product SEL and the tile's number in it for virtual block id V; tile origin of tile number V of product Q (as in the
// 256 x 256 kernel)
#define PRODUCT_OF(V, SEL, LOCAL)                                                                       \
    {                                                                                                   \
        LOCAL = (V);                                                                                    \
        SEL = 0u;                                                                                       \
        if (LOCAL >= first_tiles) { LOCAL -= first_tiles; SEL = 1u; }                                   \
    }
#define TILE_ORIGIN(Q, V, M0, N0)                                                                       \
    {                                                                                                   \
        const uint32_t v_ = (V), tt_ = (Q).total_tiles;                                                 \
        if (v_ < tt_) {                                                                                 \
            const uint32_t per_ = tt_ >> 3, rem_ = tt_ & 7u, GM_ = (Q).band_height;                     \
            const uint32_t tiles_m_ = (Q).tiles_m, tiles_n_ = (Q).tiles_n;                              \
            const uint32_t xcd_ = v_ & 7u;                                                              \
            const uint32_t tile_ = xcd_ * per_ + (xcd_ < rem_ ? xcd_ : rem_) + (v_ >> 3);               \
            const uint32_t band_ = tile_ / (GM_ * tiles_n_);                                            \
            const uint32_t band_rows_ = (tiles_m_ - band_ * GM_) < GM_ ? (tiles_m_ - band_ * GM_) : GM_; \
            const uint32_t in_band_ = tile_ - band_ * GM_ * tiles_n_;                                   \
            M0 = (band_ * GM_ + in_band_ % band_rows_) * BM;                                            \
            N0 = (in_band_ / band_rows_) * BN;                                                          \
        } else {                                                                                        \
            M0 = (Q).m; N0 = (Q).n;                                                                     \
        }                                                                                               \
    }
    uint32_t iv = blockIdx.x, ist = 0u;                  // issue cursor: the tile and stage the next loads belong to
    v4i_t res_a, res_b, res_s;
    uint32_t kb, istages, S2i, goff, gstep, soff;        // of the cursor's product
    const uint32_t drow = wave * 16u + (lane >> 2);
    const uint32_t dcol = (lane & 3u) ^ ((drow >> 2) & 3u);
#define ISSUE_SETUP()                                                                                   \
    {                                                                                                   \
        uint32_t sel_, lv_, m0_, n0_;                                                                   \
        PRODUCT_OF(iv, sel_, lv_)                                                                       \
        const GemmProblem& q_ = batch.p[sel_];                                                          \
        TILE_ORIGIN(q_, lv_, m0_, n0_)                                                                  \
        const uint32_t k_ = q_.k, kq_ = (k_ + 255u) >> 8;                                               \
        kb = k_ >> 1;                                                                                   \
        istages = (k_ + 127u) >> 7;                                                                     \
        S2i = istages < 2u ? 2u : ((istages + 1u) & ~1u);                                               \
        goff = drow * kb + dcol * 16u;          /* + j*64*kb, + stage*64 */                             \
        gstep = 64u * kb;                                                                               \
        soff = ((stile0 + (lane >> 4)) * kq_) * 256u + (lane & 15u) * 16u;   /* + quad*256 */           \
        const uint32_t rows_a_ = (q_.m - m0_) < BM ? (q_.m - m0_) : BM, rows_b_ = (q_.n - n0_) < BN ? (q_.n - n0_) : BN; \
        res_a = make_rsrc_words(q_.a_codes + (size_t)m0_ * kb, rows_a_ * kb);                           \
        res_b = make_rsrc_words(q_.b_codes + (size_t)n0_ * kb, rows_b_ * kb);                           \
        const uint32_t srow0_ = scales_of_a ? m0_ : n0_, srows_ = scales_of_a ? rows_a_ : rows_b_;      \
        res_s = make_rsrc_words((scales_of_a ? q_.a_scales : q_.b_scales) + (size_t)(srow0_ >> 5) * kq_ * 256u, \
                                has_scales ? ((srows_ + 31u) >> 5) * kq_ * 256u : 0u);                  \
    }
    ISSUE_SETUP()

    const uint32_t lds0 = (uint32_t)(size_t)(lds_ptr_t)&lds[0];
    const uint32_t swz = (lrow >> 2) & 3u;
    const uint32_t fa_base = (wm0 + lrow) * 4u, fb_base = BM * 4u + (wn0 + lrow) * 4u;
    const uint32_t sa_base = CODES * 4u + (wm0 >> 5) * 64u + lane;             // dword index in a stage
    const uint32_t sb_base = CODES * 4u + (BM / 32u) * 64u + (wn0 >> 5) * 64u + lane;

    uint32_t sa[TM], sb[TN], ra_n[TM], rb_n[TN];
    uint4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];

// code load J (0 .. LA-1: A rows, LA .. NL-1: B rows) or the scale tiles (J == NL) of the cursor's stage into ring slot SLOT
#define ISSUE(SLOT, J)                                                                                  \
    {                                                                                                   \
        const uint32_t slot_ = lds0 + ((SLOT) * STAGE + wave * 64u) * 16u;                              \
        if ((uint32_t)(J) < NL) {                                                                       \
            const uint32_t base_ = (ist * 64u + dcol * 16u < kb) ? goff + ist * 64u : kOutOfRange;      \
            const uint32_t jj_ = (uint32_t)(J) < LA ? (uint32_t)(J) : (uint32_t)(J) - LA;               \
            lds_direct_load16((uint32_t)(J) < LA ? res_a : res_b, base_ + jj_ * gstep, slot_ + (uint32_t)(J) * 4096u); \
        } else {                                                                                        \
            lds_direct_load16(res_s, (ist < istages) ? soff + (ist >> 1) * 256u : kOutOfRange, slot_ + CODES * 16u); \
        }                                                                                               \
    }
#define ISSUE_ADVANCE()                                                                                 \
    {                                                                                                   \
        ++ist;                                                                                          \
        if (ist == S2i) {                                                                               \
            ist = 0u;                                                                                   \
            iv += G;                                                                                    \
            ISSUE_SETUP()                                                                               \
        }                                                                                               \
    }
// fragment number RR of K-step S: B0 .. B(TN-1), then A0 .. A(TM-1)
#define READ_FRAG(SLOT, S, FA, FB, RR)                                                                  \
    {                                                                                                   \
        const int rr_ = (RR);                                                                           \
        if (rr_ < TN) FB[rr_] = lds[(SLOT) * STAGE + fb_base + rr_ * 128u + ((2u * (S) + lhalf) ^ swz)]; \
        else if (rr_ < R) FA[rr_ - TN] = lds[(SLOT) * STAGE + fa_base + (rr_ - TN) * 128u + ((2u * (S) + lhalf) ^ swz)]; \
    }
// the next stage's first fragments in the order the first instructions need them: A0, B0 .. B(TN-1), A1 .. A(TM-1)
#define READ_FRAG_NEXT(SLOT, FA, FB, RR)                                                                \
    {                                                                                                   \
        const int rn_ = (RR);                                                                           \
        READ_FRAG(SLOT, 0u, FA, FB, rn_ == 0 ? TN : (rn_ <= TN ? rn_ - 1 : rn_))                        \
    }
#define FENCE() __builtin_amdgcn_sched_barrier(0);
// scale dwords of a K-quad: read right behind the barrier, used behind the pair's last matrix-core instruction (see the
// 256 x 256 kernel)
#define READ_SCALES(SLOT)                                                                               \
    {                                                                                                   \
        const uint32_t* sbuf_ = reinterpret_cast<const uint32_t*>(&lds[(SLOT) * STAGE]);                \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) ra_n[i] = sbuf_[sa_base + i * 64u];         \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) rb_n[j] = sbuf_[sb_base + j * 64u];         \
    }
#define USE_SCALES(ST, GK)                                                                              \
    {                                                                                                   \
        uint32_t keep_ = 0xFFFFFFFFu;                                                                   \
        if (((ST) + 2u) * 4u > (GK)) {        /* wave-uniform: only a ragged last K-quad */             \
            const uint32_t ksteps_lane = ((GK) + 1u - lhalf) >> 1;   /* K-steps in which this half-wave has a group */ \
            const uint32_t done_ = (ST) * 2u;                                                           \
            const uint32_t nv_ = ksteps_lane > done_ ? (ksteps_lane - done_ < 4u ? ksteps_lane - done_ : 4u) : 0u; \
            keep_ = nv_ >= 4u ? 0xFFFFFFFFu : ((1u << (8u * nv_)) - 1u);                                \
        }                                                                                               \
        _Pragma("unroll") for (uint32_t i = 0; i < TM; ++i) sa[i] = (ra_n[i] & keep_) | (0x7F7F7F7Fu & ~keep_); \
        _Pragma("unroll") for (uint32_t j = 0; j < TN; ++j) sb[j] = (rb_n[j] & keep_) | (0x7F7F7F7Fu & ~keep_); \
    }

    constexpr uint32_t KEEP2 = 2u * NL + 1u;           // loads of one even and one odd stage stay in flight
    constexpr uint32_t WAIT2 = 0x0F70u | (KEEP2 & 15u) | ((KEEP2 >> 4) << 14);
#pragma unroll
    for (uint32_t s0 = 0; s0 < D; ++s0) {
#pragma unroll
        for (uint32_t j = 0; j < NL; ++j) ISSUE(s0, j)
        if ((s0 & 1u) == 0u) ISSUE(s0, NL)
        ISSUE_ADVANCE()
    }
    __builtin_amdgcn_s_waitcnt(WAIT2);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int r = 0; r < R; ++r) READ_FRAG(0u, 0u, fa0, fb0, r)
    static_assert(XR >= 0 && XR <= R / 2 + 1, "the next stage's fragment reads must fit behind the barrier");
    uint32_t csel, clv;
    PRODUCT_OF(blockIdx.x, csel, clv)
    READ_SCALES(0u)
    USE_SCALES(0u, batch.p[csel].k >> 5)

// one stage: PAR = its parity, slots SL = its own, SL1 = the next stage's, SLI = the one being filled; NEXT_ST: the
// local index of the stage after the next (odd stages read its K-quad's scales)
#define STAGE_BODY(PAR, SL, SL1, SLI, NEXT_ST, NEXT_GK)                                                 \
    {                                                                                                   \
        _Pragma("unroll") for (int idx = 0; idx < 2 * NM; ++idx) {                                      \
            const int ij_ = idx % NM, I_ = ij_ / TN, J_ = ij_ % TN;                                     \
            if (idx < NM) acc[I_][J_] = mfma_fp4<2 * PAR>(fa0[I_], fb0[J_], acc[I_][J_], sa[I_], sb[J_]); \
            else acc[I_][J_] = mfma_fp4<2 * PAR + 1>(fa1[I_], fb1[J_], acc[I_][J_], sa[I_], sb[J_]);    \
            asm volatile("" : "+a"(acc[I_][J_]));                                                       \
            FENCE()                                                                                     \
            if (idx < RS_END) {                                                                         \
                _Pragma("unroll") for (int q_ = 0; q_ < RPS; ++q_) READ_FRAG(SL, 1u, fa1, fb1, idx * RPS + q_) \
                FENCE()                                                                                 \
            }                                                                                           \
            if (idx >= RS_END && idx < P) {                                                             \
                _Pragma("unroll") for (int l_ = 0; l_ < (int)NL; ++l_)                                  \
                    if (RS_END + (l_ * (P - RS_END)) / (int)NL == idx) { ISSUE(SLI, l_) FENCE() }       \
            }                                                                                           \
            if (idx == P - 1) {                                                                         \
                if (PAR == 1) { ISSUE(SLI, NL) FENCE() }   /* the stage being filled is even */         \
                ISSUE_ADVANCE()                                                                         \
                __builtin_amdgcn_s_waitcnt(WAIT2);                                                      \
                __builtin_amdgcn_s_barrier();                                                           \
                FENCE()                                                                                 \
                if (PAR == 1) { READ_SCALES(SL1) FENCE() }                                              \
            }                                                                                           \
            if (idx >= P) {         /* two reads per slot while more reads than slots are left, then one */ \
                _Pragma("unroll") for (int r_ = 0; r_ < R; ++r_)                                        \
                    if (P + (r_ < 2 * XR ? r_ / 2 : r_ - XR) == idx) READ_FRAG_NEXT(SL1, fa0, fb0, r_)  \
                FENCE()                                                                                 \
            }                                                                                           \
        }                                                                                               \
        if (PAR == 1) { USE_SCALES(NEXT_ST, NEXT_GK) FENCE() }                                          \
    }

    v16f acc[TM][TN];
    float* wbuf = reinterpret_cast<float*>(&lds[kRing * STAGE]) + wave * (TN * 256u);
    uint32_t g = 0u;                                       // stages done by this block (ring slot = g % kRing)
    for (uint32_t cv = blockIdx.x; cv < total_tiles; cv += G) {
        PRODUCT_OF(cv, csel, clv)
        const uint32_t ck = batch.p[csel].k, gk = ck >> 5, stages = (ck + 127u) >> 7;
        const uint32_t S2 = stages < 2u ? 2u : ((stages + 1u) & ~1u);
        // the tile's last pair of stages reads the first scales of the block's next tile, which may belong to the other product
        const uint32_t gk_after = (cv + G >= first_tiles && cv + G < total_tiles) ? (batch.p[1].k >> 5) : gk;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
        for (uint32_t st = 0u; st < S2; st += 2u, g += 2u) {
            const uint32_t sl = g & 3u;                    // g is even: sl is 0 or 2
            const uint32_t next_st = st + 2u < S2 ? st + 2u : 0u;
            const uint32_t next_gk = st + 2u < S2 ? gk : gk_after;
            STAGE_BODY(0, sl, sl + 1u, sl ^ 3u, 0u, 0u)
            STAGE_BODY(1, sl + 1u, sl ^ 2u, sl, next_st, next_gk)
        }
        const GemmProblem& q = batch.p[csel];
        uint32_t m0, n0;
        TILE_ORIGIN(q, clv, m0, n0)
        const uint32_t m = q.m, n = q.n, ldd = q.ldd;
        const uint32_t* __restrict__ mask = q.mask;
        const uint32_t row_base = m0 + wm0, col_base = n0 + wn0;
        const bool full = (ldd & 3u) == 0u && row_base + TM * 32u <= m && col_base + TN * 32u <= n && (!FUSED || mask != nullptr);
        if (full) store_tile_rows8<TM, TN, OUT_BF16, FUSED, true>(acc, wbuf, q.d, ldd, mask, q.alpha, row_base, col_base, m, n, lane, nb);
        else store_tile_rows8<TM, TN, OUT_BF16, FUSED, false>(acc, wbuf, q.d, ldd, mask, q.alpha, row_base, col_base, m, n, lane, nb);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // the stages issued past the last tile (zero-filled) have landed before the LDS is given back
    if (clock_counters && tid == 0) {
        const uint64_t t1 = __builtin_readcyclecounter(), w1 = __builtin_amdgcn_s_memrealtime();
        atomicAdd(reinterpret_cast<unsigned long long*>(clock_counters), (unsigned long long)(t1 - clk_t0));
        atomicAdd(reinterpret_cast<unsigned long long*>(clock_counters) + 1, (unsigned long long)(w1 - clk_w0));
    }
#undef PRODUCT_OF
#undef TILE_ORIGIN
#undef ISSUE_SETUP
#undef ISSUE
#undef ISSUE_ADVANCE
#undef READ_FRAG
#undef READ_FRAG_NEXT
#undef FENCE
#undef READ_SCALES
#undef USE_SCALES
#undef STAGE_BODY
}

static int stream_blocks() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n >= 8)
            cus = n & ~7;
        else
            cus = 8;
    }
    return cus;
}

// tile grid and band height of one product for block tiles of bm x bn
static GemmProblem make_problem(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes, const uint8_t* b_scales,
                                int64_t m, int64_t n, int64_t k, float alpha, void* d, int64_t ldd, const uint32_t* mask,
                                int64_t bm, int64_t bn) {
    GemmProblem q;
    q.a_codes = a_codes; q.a_scales = a_scales; q.b_codes = b_codes; q.b_scales = b_scales;
    q.d = d; q.mask = mask;
    q.m = (uint32_t)m; q.n = (uint32_t)n; q.k = (uint32_t)k; q.ldd = (uint32_t)ldd;
    q.alpha = alpha;
    q.tiles_m = (uint32_t)((m + bm - 1) / bm); q.tiles_n = (uint32_t)((n + bn - 1) / bn);
    q.band_height = (bm == 256 && bn == 256 && q.tiles_n >= 40u && (q.tiles_m & 1u) == 0u) ? 2u : 4u;
    if (g_forced_band > 0) q.band_height = (uint32_t)g_forced_band;
    q.total_tiles = q.tiles_m * q.tiles_n;
    return q;
}

template <bool OUT_BF16, bool FUSED>
static void launch_stream_batch_t(const GemmBatch& batch, uint32_t nb, hipStream_t st) {
    const uint32_t total = batch.p[0].total_tiles + batch.p[1].total_tiles, cus = (uint32_t)stream_blocks();
    hipLaunchKernelGGL((gemm_mxfp4_stream_kernel<OUT_BF16, FUSED>), dim3(total < cus ? total : cus), dim3(256), 0, st, batch, total,
                       nb, g_clock_counters);
}

template <bool OUT_BF16, bool FUSED>
static void launch_stream_t(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                            const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                            int64_t ldd, const uint32_t* mask, uint32_t nb, hipStream_t st) {
    GemmBatch batch;
    batch.p[0] = make_problem(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, 256, 256);
    batch.p[1] = GemmProblem{};      // no second product
    launch_stream_batch_t<OUT_BF16, FUSED>(batch, nb, st);
}

template <int TM, int TN, bool OUT_BF16, bool FUSED>
static void launch_stream_tile_batch_t(const GemmBatch& batch, uint32_t nb, hipStream_t st) {
    const uint32_t total = batch.p[0].total_tiles + batch.p[1].total_tiles, cus = (uint32_t)stream_blocks();
    hipLaunchKernelGGL((gemm_mxfp4_stream_tile_kernel<TM, TN, OUT_BF16, FUSED>), dim3(total < cus ? total : cus), dim3(256), 0, st,
                       batch, total, nb, g_clock_counters);
}

template <int TM, int TN, bool OUT_BF16, bool FUSED>
static void launch_stream_tile_t(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                                 const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                                 int64_t ldd, const uint32_t* mask, uint32_t nb, hipStream_t st) {
    GemmBatch batch;
    batch.p[0] = make_problem(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, 64 * TM, 64 * TN);
    batch.p[1] = GemmProblem{};      // no second product
    launch_stream_tile_batch_t<TM, TN, OUT_BF16, FUSED>(batch, nb, st);
}

// Variants: 0 = 256x256 tiles (hand-scheduled stage), 1 = 128x256 tiles, 2 = 128x128 tiles (stage generated from the
// tile shape); all three: one block per compute unit streams its tiles through a ring of 4 LDS stages, two stages per
// trip with the scale byte picked by op_sel.  set_gemm_plan overrides the size heuristic (tests reach every variant
// through it).
// fused != 0: D = alpha * H_along_n((A B^T) . mask) with Hadamard blocks of nb = 1, 2 or 4 groups of 32 columns (mask may
// be null = all ones), n % (32 nb) == 0.
static int pick_variant(int64_t m, int64_t n, int fused, uint32_t nb) {
    int variant = g_forced_variant;
    if (variant < 0) {
        // The tile shape that keeps most of the chip's matrix-core time useful: share of the compute-unit rounds that hold a
        // tile x what a compute unit gets out of the shape (256x256: 1; 128x256: 0.84; 128x128: 0.54 -- per-area round times
        // measured on an MI355X at K = 2048 .. 8192).  Checked against measured best shapes: 16384x4096x4096 and every other
        // product of configuration 4 -> 256x256; 5632x2048x8192 (176 big tiles, 80 units idle) -> 256x256 (58.8 us against
        // 73.2 as 128x256); 3072^3 -> 256x256; 4096x2048x2048 -> 128x256 (19.1 us against 23.0); 2048x2048x4096 -> 128x128
        // (20.5 us against 23.7 and 34.9); 1024x1024x8192 -> 128x128.
        const double cus = (double)stream_blocks();
        const double worth[3] = {1.0, 0.84, 0.54};
        const int64_t bm[3] = {256, 128, 128}, bn[3] = {256, 256, 128};
        double best = -1.0;
        for (int v = 0; v < 3; ++v) {
            const double tiles = (double)(((m + bm[v] - 1) / bm[v]) * ((n + bn[v] - 1) / bn[v]));
            const double rounds = (double)(int64_t)((tiles + cus - 1.0) / cus);
            const double score = tiles / (rounds * cus) * worth[v];
            if (score > best) { best = score; variant = v; }
        }
    }
    if (fused && nb >= 4u && variant == 2) variant = 1;   // a block of 128 columns needs the 128-column wave tile
    return variant;
}

hipError_t launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                       const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, float alpha, void* d,
                       int d_bf16, int64_t ldd, int fused, const uint32_t* mask, uint32_t nb, hipStream_t st) {
    if (m == 0 || n == 0) return hipSuccess;
    const int variant = pick_variant(m, n, fused, nb);
#define QUARTET_DISPATCH(FN, ...)                                                                     \
    do {                                                                                              \
        if (d_bf16) { if (fused) FN<__VA_ARGS__ true, true>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, nb, st); \
                      else FN<__VA_ARGS__ true, false>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, nb, st); }   \
        else { if (fused) FN<__VA_ARGS__ false, true>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, nb, st);      \
               else FN<__VA_ARGS__ false, false>(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, ldd, mask, nb, st); }         \
    } while (0)
    if (variant == 1) QUARTET_DISPATCH(launch_stream_tile_t, 2, 4, );
    else if (variant == 2) QUARTET_DISPATCH(launch_stream_tile_t, 2, 2, );
    else QUARTET_DISPATCH(launch_stream_t, );
#undef QUARTET_DISPATCH
    return hipGetLastError();
}

// Two gradient products in one launch (both with the fused epilogue, results of one type).  One tile shape serves both: the
// one with the smallest estimated time of the busiest block, which walks the virtual tile ids b, b + G, ... over the first
// product's tiles and then the second's; a tile costs its inner dimension plus the epilogue (about 1100 elements' worth of
// stages), times the shape's area, over the shape's efficiency (pick_variant's figures).
hipError_t launch_gemm_grad_pair(const GemmArgs& g0, const GemmArgs& g1, int d_bf16, uint32_t nb, hipStream_t st) {
    const bool empty0 = g0.m == 0 || g0.n == 0, empty1 = g1.m == 0 || g1.n == 0;
    if (empty0 || empty1) {
        hipError_t e = launch_gemm(g0.a_codes, g0.a_scales, g0.b_codes, g0.b_scales, g0.m, g0.n, g0.k, g0.alpha, g0.d, d_bf16, g0.ldd,
                                   1, g0.mask, nb, st);
        if (e != hipSuccess) return e;
        return launch_gemm(g1.a_codes, g1.a_scales, g1.b_codes, g1.b_scales, g1.m, g1.n, g1.k, g1.alpha, g1.d, d_bf16, g1.ldd, 1,
                           g1.mask, nb, st);
    }
    const int64_t bm[3] = {256, 128, 128}, bn[3] = {256, 256, 128};
    int variant = g_forced_variant;
    if (variant < 0) {
        const double cost_per_area[3] = {1.0, 0.5 / 0.84, 0.25 / 0.54};
        const int64_t cus = stream_blocks();
        double best = -1.0;
        for (int v = 0; v < 3; ++v) {
            const int64_t t0 = ((g0.m + bm[v] - 1) / bm[v]) * ((g0.n + bn[v] - 1) / bn[v]);
            const int64_t t1 = ((g1.m + bm[v] - 1) / bm[v]) * ((g1.n + bn[v] - 1) / bn[v]);
            const int64_t blocks = t0 + t1 < cus ? t0 + t1 : cus;
            double busiest = 0.0;
            for (int64_t b = 0; b < blocks; ++b) {
                const int64_t n0 = t0 > b ? (t0 - b + blocks - 1) / blocks : 0;
                const int64_t upto = t0 + t1 - 1, before = t0 - 1;     // ids congruent to b up to these, inclusive
                const int64_t n1 = (upto >= b ? (upto - b) / blocks + 1 : 0) - (before >= b ? (before - b) / blocks + 1 : 0);
                const double load = (double)n0 * (double)(g0.k + 1100) + (double)n1 * (double)(g1.k + 1100);
                if (load > busiest) busiest = load;
            }
            const double t = busiest * cost_per_area[v];
            if (best < 0.0 || t < best) { best = t; variant = v; }
        }
    }
    if (nb >= 4u && variant == 2) variant = 1;   // a block of 128 columns needs the 128-column wave tile
    GemmBatch batch;
    batch.p[0] = make_problem(g0.a_codes, g0.a_scales, g0.b_codes, g0.b_scales, g0.m, g0.n, g0.k, g0.alpha, g0.d, g0.ldd, g0.mask,
                              bm[variant], bn[variant]);
    batch.p[1] = make_problem(g1.a_codes, g1.a_scales, g1.b_codes, g1.b_scales, g1.m, g1.n, g1.k, g1.alpha, g1.d, g1.ldd, g1.mask,
                              bm[variant], bn[variant]);
    if (variant == 1) { if (d_bf16) launch_stream_tile_batch_t<2, 4, true, true>(batch, nb, st); else launch_stream_tile_batch_t<2, 4, false, true>(batch, nb, st); }
    else if (variant == 2) { if (d_bf16) launch_stream_tile_batch_t<2, 2, true, true>(batch, nb, st); else launch_stream_tile_batch_t<2, 2, false, true>(batch, nb, st); }
    else { if (d_bf16) launch_stream_batch_t<true, true>(batch, nb, st); else launch_stream_batch_t<false, true>(batch, nb, st); }
    return hipGetLastError();
}

}  // namespace quartet
