// C ABI of the Quartet MXFP4 library: argument validation and kernel sequencing only.
// Declarations, argument meaning and citations are in include/quartet.h.
#include "../../include/quartet.h"

#include <hip/hip_runtime.h>

#include "device_common.h"
#include "launchers.h"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return QUARTET_EHIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Philox4x32-10 on the host (Salmon et al., SC'11), used only to derive the sign word.
void philox_host(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

constexpr int64_t kMaxGroups = (int64_t)1 << 31;


// shape checks shared by the quantizers; returns QUARTET_OK or an error
int check_quant_shape(int64_t rows, int64_t k, int64_t ldx, int transpose) {
    if (rows < 0 || k < 0 || (k % 32) != 0) return QUARTET_EINVAL;
    if (transpose != 0 && transpose != 1) return QUARTET_EINVAL;
    if ((ldx % 8) != 0 || ldx < (transpose ? rows : k)) return QUARTET_EINVAL;
    if (transpose && (rows % 8) != 0) return QUARTET_EINVAL;
    if (rows > 0 && (k / 32) > kMaxGroups / (rows > 0 ? rows : 1)) return QUARTET_ENOTSUP;
    if (rows * (k / 32) >= kMaxGroups) return QUARTET_ENOTSUP;
    if ((k + 255) / 256 > 65535) return QUARTET_ENOTSUP;
    // a block's corner of the source (8 rows; 256 rows when transposed) must fit a 32-bit byte range
    if (ldx >= ((int64_t)1 << (transpose ? 22 : 27))) return QUARTET_ENOTSUP;
    return QUARTET_OK;
}

// Hadamard block in elements -> groups per block (0 if unsupported)
uint32_t block_groups(int hb) { return (hb == 32 || hb == 64 || hb == 128 || hb == 256) ? (uint32_t)hb / 32u : 0u; }

quartet::SrParams make_params(uint32_t nb, const uint32_t* sign_words, uint64_t seed, uint32_t stream_id) {
    quartet::SrParams p = {};
    p.nb = nb;
    p.key0 = (uint32_t)seed;
    p.key1 = (uint32_t)(seed >> 32);
    p.stream_id = stream_id;
    for (uint32_t j = 0; j < 8u; ++j) p.sign_words[j] = (sign_words && j < nb) ? sign_words[j] : 0u;
    p.sign_word = p.sign_words[0];
    return p;
}

// ---- optional launch profiling: a pair of events around every kernel launch of the library
struct ProfileState {
    bool enabled = false;
    int capacity = 0, count = 0;
    unsigned kinds = ~0u;   // bit i set: launches of kind i are recorded
    hipEvent_t* start = nullptr;
    hipEvent_t* stop = nullptr;
    int* kind = nullptr;
};
ProfileState g_prof;

struct ProfileScope {
    int slot = -1;
    hipStream_t st;
    ProfileScope(int kind, hipStream_t s) : st(s) {
        if (g_prof.enabled && ((g_prof.kinds >> kind) & 1u) && g_prof.count < g_prof.capacity) {
            slot = g_prof.count++;
            g_prof.kind[slot] = kind;
            (void)hipEventRecord(g_prof.start[slot], st);
        }
    }
    ~ProfileScope() {
        if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], st);
    }
};

void profile_free() {
    for (int i = 0; i < g_prof.capacity; ++i) {
        (void)hipEventDestroy(g_prof.start[i]);
        (void)hipEventDestroy(g_prof.stop[i]);
    }
    delete[] g_prof.start; delete[] g_prof.stop; delete[] g_prof.kind;
    const unsigned kinds = g_prof.kinds;
    g_prof = ProfileState();
    g_prof.kinds = kinds;
}

size_t align256(size_t x) { return (x + 255u) & ~(size_t)255u; }

size_t scale_bytes(int64_t rows, int64_t k) {
    return (size_t)((rows + 31) / 32) * (size_t)((k + 255) / 256) * 256u;
}

struct BwdWorkspace {
    size_t g_codes, g_scales;       // dy quantized along out            [tokens x out]
    size_t gt_codes, gt_scales;     // dy^T quantized along the tokens   [out x tokens]
    size_t bw_codes, bw_scales;     // W_q re-quantized along out        [in x out]
    size_t bx_codes, bx_scales;     // X_q re-quantized along the tokens [in x tokens]
    size_t acc, total;
};

// All four operands of the two gradient products have room of their own (the three that do not feed the first product
// are converted in one launch while it still waits).  with_acc: room for the fp32 product of the larger gradient GEMM
// (Hadamard blocks above 128 apply the gradient epilogue in a kernel of its own).
BwdWorkspace plan_bwd(int64_t tokens, int64_t in, int64_t out, bool with_acc = false) {
    BwdWorkspace w;
    const size_t to = (size_t)tokens * (size_t)out;
    size_t off = 0;
    w.g_codes = off; off += align256(to / 2);
    w.g_scales = off; off += align256(scale_bytes(tokens, out));
    w.gt_codes = off; off += align256(to / 2);
    w.gt_scales = off; off += align256(scale_bytes(out, tokens));
    w.bw_codes = off; off += align256((size_t)in * (size_t)out / 2);
    w.bw_scales = off; off += align256(scale_bytes(in, out));
    w.bx_codes = off; off += align256((size_t)in * (size_t)tokens / 2);
    w.bx_scales = off; off += align256(scale_bytes(in, tokens));
    w.acc = off;
    if (with_acc) off += align256(sizeof(float) * (size_t)in * (size_t)(out > tokens ? out : tokens));
    w.total = off;
    return w;
}

// ---- workspace of quartet_linear_bwd_static: device memory that exists from the moment the library is loaded, one copy
// per GPU.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
constexpr size_t kStaticScratchBytes = QUARTET_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (resolved once per device, with that device current).
int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return QUARTET_ENOTSUP;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return QUARTET_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return QUARTET_OK;
}

}  // namespace

using quartet::SrParams;

extern "C" {

int quartet_last_hip_error(void) { return g_last_hip_error; }

int quartet_sr_bits(void) { return 22; }

size_t quartet_scale_bytes(int64_t rows, int64_t k) {
    if (rows < 0 || k < 0) return 0;
    return scale_bytes(rows, k);
}

int quartet_profile_enable(int max_records) {
    profile_free();
    if (max_records < 0) return QUARTET_EINVAL;
    if (max_records == 0) return QUARTET_OK;
    g_prof.start = new hipEvent_t[max_records];
    g_prof.stop = new hipEvent_t[max_records];
    g_prof.kind = new int[max_records];
    for (int i = 0; i < max_records; ++i) {
        // timing only: no system-scope fence (cache write-back) when an event completes
        hipError_t e = hipEventCreateWithFlags(&g_prof.start[i], hipEventDisableSystemFence);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&g_prof.stop[i], hipEventDisableSystemFence);
        if (e != hipSuccess) {
            g_prof.capacity = i;
            profile_free();
            return hip_fail(e);
        }
        g_prof.capacity = i + 1;
    }
    g_prof.enabled = true;
    return QUARTET_OK;
}

int quartet_profile_kinds(unsigned kind_mask) {
    g_prof.kinds = kind_mask;
    return QUARTET_OK;
}

int quartet_profile_read(int* kinds, float* ms, int capacity) {
    if (capacity < 0 || (capacity > 0 && (!kinds || !ms))) return QUARTET_EINVAL;
    int n = g_prof.count < capacity ? g_prof.count : capacity;
    for (int i = 0; i < n; ++i) {
        hipError_t e = hipEventSynchronize(g_prof.stop[i]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms[i], g_prof.start[i], g_prof.stop[i]);
        if (e != hipSuccess) return hip_fail(e);
        kinds[i] = g_prof.kind[i];
    }
    g_prof.count = 0;
    return n;
}

int quartet_profile_clock(uint64_t* device_counters) {
    if (reinterpret_cast<uintptr_t>(device_counters) & 7u) return QUARTET_EINVAL;
    quartet::set_clock_counters(device_counters);
    return QUARTET_OK;
}

int quartet_wall_clock_khz(void) {
    int dev = 0, khz = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    if (e != hipSuccess) return hip_fail(e);
    return khz;
}

int quartet_probe_mfma_ceiling(const uint8_t* codes, const uint8_t* scales, int64_t iterations, int blocks, float* sink,
                               uint64_t* device_counters, void* stream) {
    if (!codes || !scales || !sink) return QUARTET_EINVAL;
    if (!aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return QUARTET_EINVAL;
    if (reinterpret_cast<uintptr_t>(device_counters) & 7u) return QUARTET_EINVAL;
    if (iterations < 0 || iterations > 0x7FFFFFFF || blocks < 0 || blocks > (1 << 20)) return QUARTET_EINVAL;
    hipError_t e = quartet::launch_mfma_ceiling(codes, scales, (uint32_t)iterations, (uint32_t)blocks, sink, device_counters,
                                                (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

uint32_t quartet_sign_word(uint64_t seed) {
    const uint32_t ctr[4] = {0u, 0u, 0u, 0xFFFFFFFFu};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    philox_host(ctr, key, w);
    return w[0];
}

int quartet_sign_words(uint64_t seed, uint32_t* out8) {
    if (!out8) return QUARTET_EINVAL;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (uint32_t c = 0; c < 2u; ++c) {
        const uint32_t ctr[4] = {c, 0u, 0u, 0xFFFFFFFFu};
        philox_host(ctr, key, out8 + 4 * c);
    }
    return QUARTET_OK;
}

int quartet_quant_fwd(const void* x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                      uint8_t* codes, uint8_t* scales, uint32_t* mask, void* stream) {
    return quartet_quant_fwd_block(x_bf16, rows, k, ldx, transpose, 32, codes, scales, mask, stream);
}

int quartet_quant_fwd_block(const void* x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose, int hadamard_block,
                            uint8_t* codes, uint8_t* scales, uint32_t* mask, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u || k < 0 || (k % hadamard_block) != 0) return QUARTET_EINVAL;
    if (!x_bf16 || !codes || !scales) return QUARTET_EINVAL;
    if (!aligned16(x_bf16) || !aligned16(codes) || (mask && !aligned16(mask))) return QUARTET_EINVAL;
    if (reinterpret_cast<uintptr_t>(scales) & 3u) return QUARTET_EINVAL;
    int rc = check_quant_shape(rows, k, ldx, transpose);
    if (rc) return rc;
    SrParams p = make_params(nb, nullptr, 0u, 0u);
    ProfileScope prof(QUARTET_KIND_QUANT_FWD, (hipStream_t)stream);
    hipError_t e = quartet::launch_quant(quartet::kFwd, x_bf16, rows, k, ldx, transpose, p, codes, scales,
                                         mask, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_quant_bwd_sr(const void* x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                         uint32_t sign_word, uint64_t seed, uint32_t stream_id, int rounding,
                         uint8_t* codes, uint8_t* scales, void* stream) {
    return quartet_quant_bwd_sr_block(x_bf16, rows, k, ldx, transpose, 32, &sign_word, seed, stream_id, rounding, codes,
                                      scales, stream);
}

int quartet_quant_bwd_sr_block(const void* x_bf16, int64_t rows, int64_t k, int64_t ldx, int transpose,
                               int hadamard_block, const uint32_t* sign_words, uint64_t seed, uint32_t stream_id,
                               int rounding, uint8_t* codes, uint8_t* scales, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u || !sign_words || k < 0 || (k % hadamard_block) != 0) return QUARTET_EINVAL;
    if (!x_bf16 || !codes || !scales) return QUARTET_EINVAL;
    if (!aligned16(x_bf16) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return QUARTET_EINVAL;
    if (rounding != QUARTET_ROUND_STOCHASTIC && rounding != QUARTET_ROUND_NEAREST) return QUARTET_EINVAL;
    int rc = check_quant_shape(rows, k, ldx, transpose);
    if (rc) return rc;
    SrParams p = make_params(nb, sign_words, seed, stream_id);
    int mode = rounding == QUARTET_ROUND_NEAREST ? quartet::kBwdRtn : quartet::kBwdSr;
    ProfileScope prof(QUARTET_KIND_QUANT_BWD, (hipStream_t)stream);
    hipError_t e = quartet::launch_quant(mode, x_bf16, rows, k, ldx, transpose, p, codes, scales, nullptr,
                                         (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_requant_transpose_sr(const uint8_t* src_codes, const uint8_t* src_scales,
                                 int64_t rows, int64_t k, uint32_t sign_word, uint64_t seed,
                                 uint32_t stream_id, int rounding,
                                 uint8_t* codes, uint8_t* scales, void* stream) {
    return quartet_requant_transpose_sr_block(src_codes, src_scales, rows, k, 32, &sign_word, seed, stream_id, rounding,
                                              codes, scales, stream);
}

int quartet_fwd_operands(const void* x_bf16, const void* w_bf16, int64_t tokens, int64_t in, int64_t out,
                         uint8_t* xq_codes, uint8_t* xq_scales, uint32_t* x_mask,
                         uint8_t* wq_codes, uint8_t* wq_scales, uint32_t* w_mask, void* stream) {
    if (!x_bf16 || !w_bf16 || !xq_codes || !xq_scales || !x_mask || !wq_codes || !wq_scales || !w_mask) return QUARTET_EINVAL;
    if (!aligned16(x_bf16) || !aligned16(w_bf16) || !aligned16(xq_codes) || !aligned16(wq_codes) || !aligned16(x_mask) ||
        !aligned16(w_mask))
        return QUARTET_EINVAL;
    if ((reinterpret_cast<uintptr_t>(xq_scales) | reinterpret_cast<uintptr_t>(wq_scales)) & 3u) return QUARTET_EINVAL;
    if (in < 0 || (in % 32) != 0) return QUARTET_EINVAL;
    int rc = check_quant_shape(tokens, in, in, 0);
    if (!rc) rc = check_quant_shape(out, in, in, 0);
    if (rc) return rc;
    SrParams p = make_params(1u, nullptr, 0u, 0u);
    ProfileScope prof(QUARTET_KIND_QUANT_FWD, (hipStream_t)stream);
    hipError_t e = quartet::launch_fwd_operands(x_bf16, tokens, w_bf16, out, in, xq_codes, xq_scales, x_mask, wq_codes, wq_scales,
                                                w_mask, p, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

// The backward pass's operand conversions in one launch: dy^T, X_q^T, W_q^T, and with g_codes != null also dy itself in
// row mode (Philox stream 0).
static int bwd_operands_launch(const void* dy_bf16, int64_t tokens, int64_t in, int64_t out,
                               const uint8_t* xq_codes, const uint8_t* xq_scales, const uint8_t* wq_codes, const uint8_t* wq_scales,
                               uint32_t sign_word, uint64_t seed, int rounding,
                               uint8_t* dyt_codes, uint8_t* dyt_scales, uint8_t* xt_codes, uint8_t* xt_scales,
                               uint8_t* wt_codes, uint8_t* wt_scales, uint8_t* g_codes, uint8_t* g_scales, void* stream) {
    if (!dy_bf16 || !xq_codes || !xq_scales || !wq_codes || !wq_scales) return QUARTET_EINVAL;
    if (!dyt_codes || !dyt_scales || !xt_codes || !xt_scales || !wt_codes || !wt_scales) return QUARTET_EINVAL;
    if (!aligned16(dy_bf16) || !aligned16(xq_codes) || !aligned16(wq_codes) || !aligned16(dyt_codes) || !aligned16(xt_codes) ||
        !aligned16(wt_codes))
        return QUARTET_EINVAL;
    if ((reinterpret_cast<uintptr_t>(dyt_scales) | reinterpret_cast<uintptr_t>(xt_scales) | reinterpret_cast<uintptr_t>(wt_scales)) & 3u)
        return QUARTET_EINVAL;
    if (g_codes && (!g_scales || !aligned16(g_codes) || (reinterpret_cast<uintptr_t>(g_scales) & 3u))) return QUARTET_EINVAL;
    if (rounding != QUARTET_ROUND_STOCHASTIC && rounding != QUARTET_ROUND_NEAREST) return QUARTET_EINVAL;
    if (tokens < 0 || in < 0 || out < 0 || (tokens % 32) != 0 || (in % 32) != 0 || (out % 32) != 0) return QUARTET_EINVAL;
    // the checks of the calls this launch stands for
    int rc = check_quant_shape(out, tokens, out, 1);
    if (!rc) rc = check_quant_shape(in, tokens, in, 1);
    if (!rc) rc = check_quant_shape(in, out, in, 1);
    if (!rc && g_codes) rc = check_quant_shape(tokens, out, out, 0);
    if (!rc && in >= ((int64_t)1 << 24)) rc = QUARTET_ENOTSUP;
    if (rc) return rc;
    const int mode = rounding == QUARTET_ROUND_NEAREST ? quartet::kBwdRtn : quartet::kBwdSr;
    ProfileScope prof(QUARTET_KIND_QUANT_BWD, (hipStream_t)stream);
    hipError_t e = quartet::launch_bwd_operands(mode, dy_bf16, tokens, in, out, xq_codes, xq_scales, wq_codes, wq_scales,
                                                make_params(1u, &sign_word, seed, 2u), make_params(1u, &sign_word, seed, 3u),
                                                make_params(1u, &sign_word, seed, 1u), dyt_codes, dyt_scales, xt_codes, xt_scales,
                                                wt_codes, wt_scales, make_params(1u, &sign_word, seed, 0u), g_codes, g_scales,
                                                (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_bwd_operands(const void* dy_bf16, int64_t tokens, int64_t in, int64_t out,
                         const uint8_t* xq_codes, const uint8_t* xq_scales, const uint8_t* wq_codes, const uint8_t* wq_scales,
                         uint32_t sign_word, uint64_t seed, int rounding,
                         uint8_t* dyt_codes, uint8_t* dyt_scales, uint8_t* xt_codes, uint8_t* xt_scales,
                         uint8_t* wt_codes, uint8_t* wt_scales, void* stream) {
    return bwd_operands_launch(dy_bf16, tokens, in, out, xq_codes, xq_scales, wq_codes, wq_scales, sign_word, seed, rounding,
                               dyt_codes, dyt_scales, xt_codes, xt_scales, wt_codes, wt_scales, nullptr, nullptr, stream);
}

int quartet_requant_transpose_sr_block(const uint8_t* src_codes, const uint8_t* src_scales,
                                       int64_t rows, int64_t k, int hadamard_block, const uint32_t* sign_words,
                                       uint64_t seed, uint32_t stream_id, int rounding,
                                       uint8_t* codes, uint8_t* scales, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u || !sign_words || k < 0 || (k % hadamard_block) != 0) return QUARTET_EINVAL;
    if (!src_codes || !src_scales || !codes || !scales) return QUARTET_EINVAL;
    if (!aligned16(src_codes) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return QUARTET_EINVAL;
    if (rounding != QUARTET_ROUND_STOCHASTIC && rounding != QUARTET_ROUND_NEAREST) return QUARTET_EINVAL;
    if (rows < 0 || (rows % 32) != 0) return QUARTET_EINVAL;
    if (rows >= ((int64_t)1 << 24)) return QUARTET_ENOTSUP;   // 256 source rows of rows/2 bytes must fit a 32-bit byte range
    int rc = check_quant_shape(rows, k, (rows + 7) / 8 * 8, 1);
    if (rc) return rc;
    SrParams p = make_params(nb, sign_words, seed, stream_id);
    int mode = rounding == QUARTET_ROUND_NEAREST ? quartet::kBwdRtn : quartet::kBwdSr;
    ProfileScope prof(QUARTET_KIND_REQUANT, (hipStream_t)stream);
    hipError_t e = quartet::launch_requant_transpose(mode, src_codes, src_scales, rows, k, p, codes, scales,
                                                     (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

static int check_gemm_args(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                           const uint8_t* b_scales, int64_t m, int64_t n, int64_t k, const void* d, int d_dtype,
                           int64_t ldd) {
    if (!a_codes || !a_scales || !b_codes || !b_scales || !d) return QUARTET_EINVAL;
    if (!aligned16(a_codes) || !aligned16(b_codes) || !aligned16(d)) return QUARTET_EINVAL;
    if (m < 0 || n < 0 || k < 0 || (k % 32) != 0 || ldd < n) return QUARTET_EINVAL;
    if (ldd > ((int64_t)1 << 21)) return QUARTET_ENOTSUP;
    if (d_dtype != QUARTET_DTYPE_F32 && d_dtype != QUARTET_DTYPE_BF16) return QUARTET_EINVAL;
    if (m >= ((int64_t)1 << 31) || n >= ((int64_t)1 << 31) || k > ((int64_t)1 << 23)) return QUARTET_ENOTSUP;
    if (((m + 127) / 128) * ((n + 127) / 128) >= ((int64_t)1 << 31)) return QUARTET_ENOTSUP;
    if ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(b_scales)) & 3u) return QUARTET_EINVAL;
    return QUARTET_OK;
}

int quartet_mxfp4_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                       const uint8_t* b_codes, const uint8_t* b_scales,
                       int64_t m, int64_t n, int64_t k, float alpha,
                       void* d, int d_dtype, int64_t ldd, void* stream) {
    int rc = check_gemm_args(a_codes, a_scales, b_codes, b_scales, m, n, k, d, d_dtype, ldd);
    if (rc) return rc;
    ProfileScope prof(QUARTET_KIND_GEMM, (hipStream_t)stream);
    hipError_t e = quartet::launch_gemm(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d,
                                        d_dtype == QUARTET_DTYPE_BF16, ldd, 0, nullptr, 1u, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_debug_set_gemm_plan(int variant, int band_height) {
    if (variant < -1 || variant > 2 || band_height < 0 || band_height > 64) return QUARTET_EINVAL;
    quartet::set_gemm_plan(variant, band_height);
    return QUARTET_OK;
}

int quartet_mxfp4_gemm_grad(const uint8_t* a_codes, const uint8_t* a_scales,
                            const uint8_t* b_codes, const uint8_t* b_scales,
                            int64_t m, int64_t n, int64_t k, const uint32_t* mask, float scale,
                            void* d, int d_dtype, int64_t ldd, void* stream) {
    return quartet_mxfp4_gemm_grad_block(a_codes, a_scales, b_codes, b_scales, m, n, k, 32, mask, scale, d, d_dtype, ldd,
                                         stream);
}

int quartet_mxfp4_gemm_grad_block(const uint8_t* a_codes, const uint8_t* a_scales,
                                  const uint8_t* b_codes, const uint8_t* b_scales,
                                  int64_t m, int64_t n, int64_t k, int hadamard_block, const uint32_t* mask,
                                  float scale, void* d, int d_dtype, int64_t ldd, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u) return QUARTET_EINVAL;
    if (nb > 4u) return QUARTET_ENOTSUP;     // a block of 256 columns spans two waves' tiles: plain GEMM + quartet_grad_epilogue_block
    int rc = check_gemm_args(a_codes, a_scales, b_codes, b_scales, m, n, k, d, d_dtype, ldd);
    if (rc) return rc;
    if ((n % hadamard_block) != 0) return QUARTET_EINVAL;
    if (mask && (reinterpret_cast<uintptr_t>(mask) & 3u)) return QUARTET_EINVAL;
    ProfileScope prof(QUARTET_KIND_GEMM, (hipStream_t)stream);
    hipError_t e = quartet::launch_gemm(a_codes, a_scales, b_codes, b_scales, m, n, k, scale, d,
                                        d_dtype == QUARTET_DTYPE_BF16, ldd, 1, mask, nb, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

static int check_gemm_grad_args(const quartet_gemm_grad_args* g, int d_dtype, int hadamard_block) {
    if (!g) return QUARTET_EINVAL;
    int rc = check_gemm_args(g->a_codes, g->a_scales, g->b_codes, g->b_scales, g->m, g->n, g->k, g->d, d_dtype, g->ldd);
    if (rc) return rc;
    if ((g->n % hadamard_block) != 0) return QUARTET_EINVAL;
    if (g->mask && (reinterpret_cast<uintptr_t>(g->mask) & 3u)) return QUARTET_EINVAL;
    return QUARTET_OK;
}

// both products with Hadamard blocks of hadamard_block = 32, 64 or 128 columns
static int gemm_grad_pair_block(const quartet_gemm_grad_args* first, const quartet_gemm_grad_args* second, int hadamard_block,
                                int d_dtype, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u || nb > 4u) return QUARTET_EINVAL;
    int rc = check_gemm_grad_args(first, d_dtype, hadamard_block);
    if (rc) return rc;
    rc = check_gemm_grad_args(second, d_dtype, hadamard_block);
    if (rc) return rc;
    const quartet::GemmArgs g0 = {first->a_codes, first->a_scales, first->b_codes, first->b_scales, first->m, first->n, first->k,
                                  first->scale, first->d, first->ldd, first->mask};
    const quartet::GemmArgs g1 = {second->a_codes, second->a_scales, second->b_codes, second->b_scales, second->m, second->n,
                                  second->k, second->scale, second->d, second->ldd, second->mask};
    ProfileScope prof(QUARTET_KIND_GEMM, (hipStream_t)stream);
    hipError_t e = quartet::launch_gemm_grad_pair(g0, g1, d_dtype == QUARTET_DTYPE_BF16, nb, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_mxfp4_gemm_grad_pair(const quartet_gemm_grad_args* first, const quartet_gemm_grad_args* second, int d_dtype,
                                 void* stream) {
    return gemm_grad_pair_block(first, second, 32, d_dtype, stream);
}

int quartet_mxfp8_quant(const void* x_bf16, int64_t rows, int64_t k, int64_t ldx,
                        uint8_t* codes, uint8_t* scales, void* stream) {
    if (!x_bf16 || !codes || !scales) return QUARTET_EINVAL;
    if (!aligned16(x_bf16) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return QUARTET_EINVAL;
    int rc = check_quant_shape(rows, k, ldx, 0);
    if (rc) return rc;
    ProfileScope prof(QUARTET_KIND_FP8_QUANT, (hipStream_t)stream);
    hipError_t e = quartet::launch_mxfp8_quant(x_bf16, rows, k, ldx, codes, scales, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_mxfp8_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                       const uint8_t* b_codes, const uint8_t* b_scales,
                       int64_t m, int64_t n, int64_t k, float alpha,
                       void* d, int d_dtype, int64_t ldd, void* stream) {
    int rc = check_gemm_args(a_codes, a_scales, b_codes, b_scales, m, n, k, d, d_dtype, ldd);
    if (rc) return rc;
    ProfileScope prof(QUARTET_KIND_FP8_GEMM, (hipStream_t)stream);
    hipError_t e = quartet::launch_mxfp8_gemm(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d,
                                              d_dtype == QUARTET_DTYPE_BF16, ldd, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_grad_epilogue(const float* g, const uint32_t* mask, int64_t m, int64_t n, float scale,
                          void* out, int out_dtype, void* stream) {
    return quartet_grad_epilogue_block(g, mask, m, n, 32, scale, out, out_dtype, stream);
}

int quartet_grad_epilogue_block(const float* g, const uint32_t* mask, int64_t m, int64_t n, int hadamard_block,
                                float scale, void* out, int out_dtype, void* stream) {
    const uint32_t nb = block_groups(hadamard_block);
    if (nb == 0u || n < 0 || (n % hadamard_block) != 0) return QUARTET_EINVAL;
    if (!g || !out) return QUARTET_EINVAL;
    if (!aligned16(g) || !aligned16(out)) return QUARTET_EINVAL;
    if (m < 0 || n < 0 || (n % 32) != 0) return QUARTET_EINVAL;
    if (out_dtype != QUARTET_DTYPE_F32 && out_dtype != QUARTET_DTYPE_BF16) return QUARTET_EINVAL;
    if (out_dtype == QUARTET_DTYPE_BF16 && out == (const void*)g) return QUARTET_EINVAL;
    if (m > 0 && (n / 32) >= kMaxGroups / m) return QUARTET_ENOTSUP;
    ProfileScope prof(QUARTET_KIND_EPILOGUE, (hipStream_t)stream);
    hipError_t e = quartet::launch_grad_epilogue(g, mask, m, n, nb, scale, out, out_dtype == QUARTET_DTYPE_BF16,
                                                 (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_mxfp4_dequant(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t k,
                          float* out, void* stream) {
    if (!codes || !scales || !out) return QUARTET_EINVAL;
    if (!aligned16(codes) || !aligned16(out)) return QUARTET_EINVAL;
    if (rows < 0 || k < 0 || (k % 32) != 0) return QUARTET_EINVAL;
    ProfileScope prof(QUARTET_KIND_DEQUANT, (hipStream_t)stream);
    hipError_t e = quartet::launch_dequant(codes, scales, rows, k, out, (hipStream_t)stream);
    return e == hipSuccess ? QUARTET_OK : hip_fail(e);
}

int quartet_linear_fwd(const void* x_bf16, const void* w_bf16, int64_t tokens, int64_t in, int64_t out,
                       void* y, int y_dtype,
                       uint8_t* xq_codes, uint8_t* xq_scales, uint32_t* x_mask,
                       uint8_t* wq_codes, uint8_t* wq_scales, uint32_t* w_mask,
                       void* stream) {
    return quartet_linear_fwd_block(x_bf16, w_bf16, tokens, in, out, 32, y, y_dtype, xq_codes, xq_scales, x_mask,
                                    wq_codes, wq_scales, w_mask, stream);
}

int quartet_linear_fwd_block(const void* x_bf16, const void* w_bf16, int64_t tokens, int64_t in, int64_t out,
                             int hadamard_block, void* y, int y_dtype,
                             uint8_t* xq_codes, uint8_t* xq_scales, uint32_t* x_mask,
                             uint8_t* wq_codes, uint8_t* wq_scales, uint32_t* w_mask,
                             void* stream) {
    if (!x_bf16 || !w_bf16 || !y || !xq_codes || !xq_scales || !x_mask || !wq_codes || !wq_scales || !w_mask)
        return QUARTET_EINVAL;
    if (block_groups(hadamard_block) == 0u) return QUARTET_EINVAL;
    if (tokens < 0 || in < 0 || out < 0 || (in % hadamard_block) != 0) return QUARTET_EINVAL;
    int rc;
    if (hadamard_block == 32) {
        rc = quartet_fwd_operands(x_bf16, w_bf16, tokens, in, out, xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask, stream);
        if (rc) return rc;
    } else {
        rc = quartet_quant_fwd_block(x_bf16, tokens, in, in, 0, hadamard_block, xq_codes, xq_scales, x_mask, stream);
        if (rc) return rc;
        rc = quartet_quant_fwd_block(w_bf16, out, in, in, 0, hadamard_block, wq_codes, wq_scales, w_mask, stream);
        if (rc) return rc;
    }
    return quartet_mxfp4_gemm(xq_codes, xq_scales, wq_codes, wq_scales, tokens, out, in, 1.0f, y, y_dtype,
                              out, stream);
}

size_t quartet_linear_workspace_bytes(int64_t tokens, int64_t in, int64_t out) {
    return quartet_linear_workspace_bytes_block(tokens, in, out, 32);
}

size_t quartet_linear_workspace_bytes_block(int64_t tokens, int64_t in, int64_t out, int hadamard_block) {
    if (block_groups(hadamard_block) == 0u) return 0;
    if (tokens < 0 || in < 0 || out < 0) return 0;
    if ((tokens % hadamard_block) != 0 || (in % hadamard_block) != 0 || (out % hadamard_block) != 0) return 0;
    return plan_bwd(tokens, in, out, hadamard_block > 128).total;
}

int quartet_linear_bwd(const void* dy_bf16, int64_t tokens, int64_t in, int64_t out,
                       const uint8_t* xq_codes, const uint8_t* xq_scales, const uint32_t* x_mask,
                       const uint8_t* wq_codes, const uint8_t* wq_scales, const uint32_t* w_mask,
                       uint64_t seed, int rounding,
                       void* dx, void* dw, int grad_dtype,
                       void* workspace, size_t workspace_bytes, void* stream) {
    return quartet_linear_bwd_block(dy_bf16, tokens, in, out, 32, xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask,
                                    seed, rounding, dx, dw, grad_dtype, workspace, workspace_bytes, stream);
}

size_t quartet_static_scratch_bytes(void) { return kStaticScratchBytes; }

int quartet_linear_bwd_static(const void* dy_bf16, int64_t tokens, int64_t in, int64_t out,
                              const uint8_t* xq_codes, const uint8_t* xq_scales, const uint32_t* x_mask,
                              const uint8_t* wq_codes, const uint8_t* wq_scales, const uint32_t* w_mask,
                              uint64_t seed, int rounding,
                              void* dx, void* dw, int grad_dtype, void* stream) {
    if (!dy_bf16 || !xq_codes || !xq_scales || !x_mask || !wq_codes || !wq_scales || !w_mask || !dx || !dw)
        return QUARTET_EINVAL;
    if (tokens < 0 || in < 0 || out < 0 || (tokens % 32) != 0 || (in % 32) != 0 || (out % 32) != 0) return QUARTET_EINVAL;
    // size first (in floating point: the exact plan could overflow on absurd shapes), then the exact plan
    const double rough = 1.0625 * (double)tokens * (double)out + 0.53125 * ((double)in * (double)out + (double)in * (double)tokens);
    if (rough > (double)kStaticScratchBytes) return QUARTET_ENOTSUP;
    const size_t need = plan_bwd(tokens, in, out, false).total;
    if (need > kStaticScratchBytes) return QUARTET_ENOTSUP;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc) return rc;
    // every byte of the workspace that a kernel reads as data was written by an earlier kernel of the same call, so
    // nothing has to be cleared between calls
    return quartet_linear_bwd_block(dy_bf16, tokens, in, out, 32, xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask,
                                    seed, rounding, dx, dw, grad_dtype, ws, kStaticScratchBytes, stream);
}

int quartet_linear_bwd_block(const void* dy_bf16, int64_t tokens, int64_t in, int64_t out, int hadamard_block,
                             const uint8_t* xq_codes, const uint8_t* xq_scales, const uint32_t* x_mask,
                             const uint8_t* wq_codes, const uint8_t* wq_scales, const uint32_t* w_mask,
                             uint64_t seed, int rounding,
                             void* dx, void* dw, int grad_dtype,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!dy_bf16 || !xq_codes || !xq_scales || !x_mask || !wq_codes || !wq_scales || !w_mask || !dx || !dw)
        return QUARTET_EINVAL;
    const int hb = hadamard_block;
    if (block_groups(hb) == 0u) return QUARTET_EINVAL;
    if (tokens < 0 || in < 0 || out < 0) return QUARTET_EINVAL;
    if ((tokens % hb) != 0 || (in % hb) != 0 || (out % hb) != 0) return QUARTET_EINVAL;
    if (rounding != QUARTET_ROUND_STOCHASTIC && rounding != QUARTET_ROUND_NEAREST) return QUARTET_EINVAL;
    if (grad_dtype != QUARTET_DTYPE_F32 && grad_dtype != QUARTET_DTYPE_BF16) return QUARTET_EINVAL;
    const bool big = hb > 128;     // the GEMM applies the gradient epilogue itself for blocks up to 128
    const BwdWorkspace w = plan_bwd(tokens, in, out, big);
    if (w.total > 0 && (!workspace || workspace_bytes < w.total)) return QUARTET_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return QUARTET_EINVAL;
    uint8_t* base = static_cast<uint8_t*>(workspace);
    uint8_t *g_codes = base + w.g_codes, *g_scales = base + w.g_scales;
    uint8_t *gt_codes = base + w.gt_codes, *gt_scales = base + w.gt_scales;
    uint8_t *bw_codes = base + w.bw_codes, *bw_scales = base + w.bw_scales;
    uint8_t *bx_codes = base + w.bx_codes, *bx_scales = base + w.bx_scales;
    float* acc = reinterpret_cast<float*>(base + w.acc);
    uint32_t sw[8];
    quartet_sign_words(seed, sw);
    const float c169 = 16.0f / 9.0f;
    int rc;
    // dx = 16/9 H( (Q(dy) Q(W_q^T)^T) . M_x ), inner dimension = out   (operand streams 0, 1)
    // dW = 16/9 H( (Q(dy^T) Q(X_q^T)^T) . M_w ), inner dimension = tokens (operand streams 2, 3)
    if (hb == 32) {
        // All four operand conversions in one launch (none depends on another; every operand has its own Philox stream),
        // then both products in one launch: two launches.  Measured against Q(dy) as a launch of its own between the products:
        // +4 % on configuration 1, +2.5-5 % on 2, +0.2-2 % on 3, +0.1-0.2 % on 4.
        rc = bwd_operands_launch(dy_bf16, tokens, in, out, xq_codes, xq_scales, wq_codes, wq_scales, sw[0], seed, rounding,
                                 gt_codes, gt_scales, bx_codes, bx_scales, bw_codes, bw_scales, g_codes, g_scales, stream);
        if (rc) return rc;
        const quartet_gemm_grad_args dw_args = {gt_codes, gt_scales, bx_codes, bx_scales, out, in, tokens, w_mask, c169, dw, in};
        const quartet_gemm_grad_args dx_args = {g_codes, g_scales, bw_codes, bw_scales, tokens, in, out, x_mask, c169, dx, in};
        return quartet_mxfp4_gemm_grad_pair(&dw_args, &dx_args, grad_dtype, stream);
    }
    // wider Hadamard blocks: one launch per operand conversion
    rc = quartet_quant_bwd_sr_block(dy_bf16, out, tokens, out, 1, hb, sw, seed, 2u, rounding, gt_codes, gt_scales, stream);
    if (rc) return rc;
    rc = quartet_requant_transpose_sr_block(xq_codes, xq_scales, in, tokens, hb, sw, seed, 3u, rounding, bx_codes, bx_scales, stream);
    if (rc) return rc;
    if (!big) {
        // blocks of 64 and 128 columns: the other two conversions, then both products (epilogue inside) in one launch
        rc = quartet_quant_bwd_sr_block(dy_bf16, tokens, out, out, 0, hb, sw, seed, 0u, rounding, g_codes, g_scales, stream);
        if (rc) return rc;
        rc = quartet_requant_transpose_sr_block(wq_codes, wq_scales, in, out, hb, sw, seed, 1u, rounding, bw_codes, bw_scales, stream);
        if (rc) return rc;
        const quartet_gemm_grad_args dw_args = {gt_codes, gt_scales, bx_codes, bx_scales, out, in, tokens, w_mask, c169, dw, in};
        const quartet_gemm_grad_args dx_args = {g_codes, g_scales, bw_codes, bw_scales, tokens, in, out, x_mask, c169, dx, in};
        return gemm_grad_pair_block(&dw_args, &dx_args, hb, grad_dtype, stream);
    }
    // a block of 256 columns spans two waves' tiles: fp32 product, then the epilogue kernel
    rc = quartet_mxfp4_gemm(gt_codes, gt_scales, bx_codes, bx_scales, out, in, tokens, 1.0f, acc, QUARTET_DTYPE_F32, in, stream);
    if (rc) return rc;
    rc = quartet_grad_epilogue_block(acc, w_mask, out, in, hb, c169, dw, grad_dtype, stream);
    if (rc) return rc;
    rc = quartet_quant_bwd_sr_block(dy_bf16, tokens, out, out, 0, hb, sw, seed, 0u, rounding, g_codes, g_scales, stream);
    if (rc) return rc;
    rc = quartet_requant_transpose_sr_block(wq_codes, wq_scales, in, out, hb, sw, seed, 1u, rounding, bw_codes, bw_scales, stream);
    if (rc) return rc;
    rc = quartet_mxfp4_gemm(g_codes, g_scales, bw_codes, bw_scales, tokens, in, out, 1.0f, acc, QUARTET_DTYPE_F32, in, stream);
    if (rc) return rc;
    return quartet_grad_epilogue_block(acc, x_mask, tokens, in, hb, c169, dx, grad_dtype, stream);
}

}  // extern "C"
