"""Benchmark of the Quartet MXFP4 linear-layer path on one MI355X.

One step = forward + backward (Algorithm 1) of every linear layer of the workload, through
quartet_linear_fwd / quartet_linear_bwd, with inputs already resident in HBM.  Prints ONE JSON
line: whole-job TFLOP/s (6*T*I*O flops per layer), the roofline of the dominant kernel (the FP4
MFMA GEMM, timed by the library's per-launch HIP events inside the timed region) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP4_TFLOPS = 10100.0   # MI355X dense MXFP4 MFMA peak (256 CU x 2.4 GHz x 16384 flop/clk/CU)
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="workload: configuration 1..4")
    ap.add_argument("--rounding", type=int, default=0, help="backward rounding: 0 = stochastic, 1 = nearest")
    ap.add_argument("--hadamard-block", type=int, default=32,
                    help="Hadamard block in elements (32 = the method; 64, 128, 256: the wider rotations)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quant-sweep", action="store_true", help="accepted for older command lines: the quantizer sweep (config 5) runs by default")
    ap.add_argument("--no-quant-sweep", action="store_true", help="skip the quantizer-only sweep (config 5)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short whole-path timings of configurations 1-3")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the register-only matrix-core ceiling measurement")
    ap.add_argument("--fp8-compare", action="store_true",
                    help="also time the library's own MXFP8 GEMM and quantizer on the workload's shapes (the paper's comparison format)")
    ap.add_argument("--breakdown", action="store_true", help="print the per-kernel-kind time breakdown to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run a plain 1 GiB elementwise copy kernel (torch.mul by 1), the known-size "
                         "reference that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    return ap.parse_args()


class Layer:
    def __init__(self, q, torch, L, block=32):
        self.block = block
        t, i, o = L["tokens"], L["in_features"], L["out_features"]
        self.t, self.i, self.o, self.name = t, i, o, L["name"]
        dev = L["x"].device
        u8 = dict(dtype=torch.uint8, device=dev)
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        self.x, self.w, self.dy = L["x"], L["w"], L["dy"]
        self.y = torch.empty((t, o), **f32)
        self.xq_codes, self.xq_scales, self.x_mask = (torch.empty((t, i // 2), **u8),
                                                      torch.empty((q.quartet_scale_bytes(t, i),), **u8),
                                                      torch.empty((t, i // 32), **i32))
        self.wq_codes, self.wq_scales, self.w_mask = (torch.empty((o, i // 2), **u8),
                                                      torch.empty((q.quartet_scale_bytes(o, i),), **u8),
                                                      torch.empty((o, i // 32), **i32))
        self.dx = torch.empty((t, i), **f32)
        self.dw = torch.empty((o, i), **f32)
        self.ws_bytes = q.quartet_linear_workspace_bytes_block(t, i, o, block)
        self.flops = 6.0 * t * i * o

    def step(self, q, ws, seed, rounding):
        if self.block != 32:
            q.check(q.quartet_linear_fwd_block(self.x, self.w, self.t, self.i, self.o, self.block, self.y,
                                               q.QUARTET_DTYPE_F32, self.xq_codes, self.xq_scales, self.x_mask,
                                               self.wq_codes, self.wq_scales, self.w_mask))
            q.check(q.quartet_linear_bwd_block(self.dy, self.t, self.i, self.o, self.block, self.xq_codes,
                                               self.xq_scales, self.x_mask, self.wq_codes, self.wq_scales, self.w_mask,
                                               seed, rounding, self.dx, self.dw, q.QUARTET_DTYPE_F32, ws, self.ws_bytes))
            return
        q.check(q.quartet_linear_fwd(self.x, self.w, self.t, self.i, self.o, self.y, q.QUARTET_DTYPE_F32,
                                     self.xq_codes, self.xq_scales, self.x_mask,
                                     self.wq_codes, self.wq_scales, self.w_mask))
        q.check(q.quartet_linear_bwd(self.dy, self.t, self.i, self.o, self.xq_codes, self.xq_scales, self.x_mask,
                                     self.wq_codes, self.wq_scales, self.w_mask, seed, rounding,
                                     self.dx, self.dw, q.QUARTET_DTYPE_F32, ws, self.ws_bytes))


def cpu_baseline(config, layer=None, q=None):
    """The oracle, as it stands, on a bounded sample: the first layer of the workload with the token
    count cut so that the run takes roughly 10-30 s of CPU work.  With `layer` (the benchmark's own first
    layer) the sample is the first rows of the tensors the timed region ran on, and the HIP path's results
    on that sample are compared with the oracle's (same bar as the parity tests)."""
    import numpy as np
    import oracle
    from paper_2505_14669_amd import synth
    name, t, i, o = synth.CONFIGS[config]["layers"][0]
    budget = 3.6e11                       # multiply-adds the plain fp64 loops get through in 10-15 s on the box's 16 cores
    ts = int(min(t, max(32, (budget / (3.0 * i * o)) // 32 * 32)))
    if layer is not None:
        import torch
        host = lambda tensor: tensor.view(torch.int16).cpu().numpy().view(np.uint16)
        x, w, dy = host(layer.x[:ts]), host(layer.w), host(layer.dy[:ts])
    else:
        rng = np.random.Generator(np.random.PCG64(4242))
        x = synth.f32_to_bf16(rng.standard_t(3.0, size=(ts, i)).astype(np.float32))
        w = synth.f32_to_bf16(rng.standard_normal((o, i), dtype=np.float32) * np.float32(0.02))
        dy = synth.f32_to_bf16(rng.standard_normal((ts, o), dtype=np.float32) * np.float32(1e-3))
    t0 = time.perf_counter()
    y_ref, ctx = oracle.linear_fwd(x, w)
    dx_ref, dw_ref = oracle.linear_bwd(dy, ctx, 0, 0)
    dt = time.perf_counter() - t0
    cores = oracle.num_threads()
    # the same code on one thread, on the first tokens/cores rows of the same sample (about the same wall time)
    t1 = int(max(32, (ts // max(cores, 1)) // 32 * 32))
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        _, ctx1 = oracle.linear_fwd(x[:t1], w)
        oracle.linear_bwd(dy[:t1], ctx1, 0, 0)
        dt1 = time.perf_counter() - t0
    finally:
        oracle.set_num_threads(cores)
    # the quantizer oracle alone, on the same sample: forward rule (codes, scales, mask) and backward rule with stochastic rounding
    tq = time.perf_counter()
    oracle.quant_fwd(x)
    tq_fwd = time.perf_counter() - tq
    tq = time.perf_counter()
    oracle.quant_bwd_sr(x, 0x1234ABCD, 7, 0, 0)
    tq_bwd = time.perf_counter() - tq
    out = dict(value=6.0 * ts * i * o / dt / 1e12, unit="TFLOP/s", cores=cores, kind="oracle",
               quantizer=dict(fwd_rtn_GBps=round(2.65625 * ts * i / tq_fwd / 1e9, 3), bwd_sr_GBps=round(2.53125 * ts * i / tq_bwd / 1e9, 3),
                              cores=cores, sample=f"the sample's activations [{ts} x {i}], algorithmic bytes / wall time"),
               sample=f"layer '{name}' of config {config} with tokens cut to {ts} (in={i}, out={o}), fwd+bwd, {dt:.1f} s",
               single_thread=dict(value=6.0 * t1 * i * o / dt1 / 1e12, unit="TFLOP/s", cores=1,
                                  sample=f"the first {t1} tokens of that sample, {dt1:.1f} s"))
    if layer is not None and q is not None:
        # the HIP path on the same rows, stochastic rounding with the same seed: relative Frobenius errors
        f32 = dict(dtype=torch.float32, device=layer.x.device)
        y, dx, dw = torch.empty((ts, o), **f32), torch.empty((ts, i), **f32), torch.empty((o, i), **f32)
        ws_bytes = q.quartet_linear_workspace_bytes(ts, i, o)
        ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=layer.x.device)
        q.check(q.quartet_linear_fwd(layer.x[:ts], layer.w, ts, i, o, y, q.QUARTET_DTYPE_F32, layer.xq_codes, layer.xq_scales,
                                     layer.x_mask, layer.wq_codes, layer.wq_scales, layer.w_mask))
        q.check(q.quartet_linear_bwd(layer.dy[:ts], ts, i, o, layer.xq_codes, layer.xq_scales, layer.x_mask, layer.wq_codes,
                                     layer.wq_scales, layer.w_mask, 0, 0, dx, dw, q.QUARTET_DTYPE_F32, ws, ws_bytes))
        torch.cuda.synchronize()
        rel = lambda got, want: float(np.linalg.norm(got.cpu().numpy().astype(np.float64) - want) / np.linalg.norm(want))
        out["parity_on_sample"] = dict(y=rel(y, y_ref), dx=rel(dx, dx_ref), dw=rel(dw, dw_ref), tolerance=1e-5,
                                       what="relative Frobenius error of the HIP path against the oracle on that sample")
    return out


def quant_sweep(q, torch, synth):
    """Quantizer-only sweep (configuration 5): 10 warm-up + 50 timed launches per case over 4 rotating
    buffer sets (each pass streams from HBM, not from the 256 MB cache), every launch timed by the
    library's own HIP event pair; GB/s = algorithmic bytes / median launch time."""
    import statistics
    warm, reps, sets = 10, 50, 4
    out = []
    kinds = (ctypes.c_int * reps)()
    ms = (ctypes.c_float * reps)()
    for idx, (r, c) in enumerate(synth.QUANT_SWEEP):
        x = synth.device_quant_sweep_matrix(idx)
        xs = [x] + [x.clone() for _ in range(sets - 1)]
        codes = [torch.empty((r, c // 2), dtype=torch.uint8, device=x.device) for _ in xs]
        scales = [torch.empty((max(q.quartet_scale_bytes(r, c), q.quartet_scale_bytes(c, r)),), dtype=torch.uint8, device=x.device) for _ in xs]
        mask = [torch.empty((r, c // 32), dtype=torch.int32, device=x.device) for _ in xs]
        cases = [("fwd_rtn_row", 2.65625, lambda j: q.quartet_quant_fwd(xs[j], r, c, c, 0, codes[j], scales[j], mask[j])),
                 ("bwd_sr_row", 2.53125, lambda j: q.quartet_quant_bwd_sr(xs[j], r, c, c, 0, 0x1234ABCD, 7, 0, 0, codes[j], scales[j])),
                 ("bwd_rtn_row", 2.53125, lambda j: q.quartet_quant_bwd_sr(xs[j], r, c, c, 0, 0x1234ABCD, 7, 0, 1, codes[j], scales[j])),
                 ("bwd_sr_transposed", 2.53125, lambda j: q.quartet_quant_bwd_sr(xs[j], c, r, c, 1, 0x1234ABCD, 7, 0, 0, codes[j], scales[j])),
                 ("bwd_rtn_transposed", 2.53125, lambda j: q.quartet_quant_bwd_sr(xs[j], c, r, c, 1, 0x1234ABCD, 7, 0, 1, codes[j], scales[j]))]
        # a plain copy of the same matrix on the same box, timed the same way (torch's elementwise copy kernel; bytes read + written)
        cp_dst = [torch.empty_like(x) for _ in range(2)]
        for j in range(4):
            cp_dst[j % 2].copy_(xs[j % sets])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for j in range(20):
            cp_dst[j % 2].copy_(xs[j % sets])
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 4.0 * r * c * 20 / e0.elapsed_time(e1) / 1e6
        del cp_dst
        for name, bpe, fn in cases:
            for j in range(warm):
                q.check(fn(j % sets))
            torch.cuda.synchronize()
            q.check(q.quartet_profile_enable(reps))
            for it in range(reps):
                q.check(fn(it % sets))
            torch.cuda.synchronize()
            n = q.quartet_profile_read(kinds, ms, reps)
            q.quartet_profile_enable(0)
            if n != reps:
                raise RuntimeError(f"quantizer sweep: {n} of {reps} launches were timed")
            med, best = statistics.median(ms[:n]), min(ms[:n])
            gbs = bpe * r * c / med / 1e6
            out.append(dict(shape=[r, c], mode=name, ms_median=round(med, 4), ms_min=round(best, 4), GBps=round(gbs, 1),
                            GBps_best=round(bpe * r * c / best / 1e6, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4),
                            copy_GBps=round(copy_gbs, 1)))
        del xs, codes, scales, mask
    return out


def fp8_compare(q, torch, layers):
    """The workload's 21 GEMM shapes in MXFP4 and in MXFP8 (same tile skeleton, the matrix cores' FP8 rate is half
    the FP4 rate), random codes, fp32 results, every launch timed by the library's event pairs; and the forward
    quantizer of each format on the largest activation."""
    import statistics
    dev = "cuda:0"
    shapes = []
    for l in layers:
        shapes += [(l.t, l.o, l.i), (l.t, l.i, l.o), (l.o, l.i, l.t)]
    reps = 5
    kinds = (ctypes.c_int * reps)()
    ms = (ctypes.c_float * reps)()

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        q.check(q.quartet_profile_kinds(0xFFFFFFFF))
        q.check(q.quartet_profile_enable(reps))
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        n = q.quartet_profile_read(kinds, ms, reps)
        q.quartet_profile_enable(0)
        return statistics.median(ms[:n])

    t4 = t8 = flops = 0.0
    for (m, n, k) in shapes:
        d = torch.empty((m, n), dtype=torch.float32, device=dev)
        asc = torch.randint(120, 134, (q.quartet_scale_bytes(m, k),), dtype=torch.uint8, device=dev)
        bsc = torch.randint(120, 134, (q.quartet_scale_bytes(n, k),), dtype=torch.uint8, device=dev)
        a4 = torch.randint(0, 256, (m, k // 2), dtype=torch.uint8, device=dev)
        b4 = torch.randint(0, 256, (n, k // 2), dtype=torch.uint8, device=dev)
        t4 += timed(lambda: q.check(q.quartet_mxfp4_gemm(a4, asc, b4, bsc, m, n, k, 1.0, d, q.QUARTET_DTYPE_F32, n)))
        del a4, b4
        a8 = torch.randint(0, 0x7F, (m, k), dtype=torch.uint8, device=dev)      # no NaN codes
        b8 = torch.randint(0, 0x7F, (n, k), dtype=torch.uint8, device=dev)
        t8 += timed(lambda: q.check(q.quartet_mxfp8_gemm(a8, asc, b8, bsc, m, n, k, 1.0, d, q.QUARTET_DTYPE_F32, n)))
        del a8, b8, d
        flops += 2.0 * m * n * k
    big = max(layers, key=lambda l: l.t * l.i)
    r, c = big.t, big.i
    codes = torch.empty((r, c), dtype=torch.uint8, device=dev)
    scales = torch.empty((q.quartet_scale_bytes(r, c),), dtype=torch.uint8, device=dev)
    mask = torch.empty((r, c // 32), dtype=torch.int32, device=dev)
    tq4 = timed(lambda: q.check(q.quartet_quant_fwd(big.x, r, c, c, 0, codes, scales, mask)))
    tq8 = timed(lambda: q.check(q.quartet_mxfp8_quant(big.x, r, c, c, codes, scales)))
    return {"gemm_shapes": len(shapes),
            "gemm_mxfp4_tflops": round(flops / t4 / 1e9, 1), "gemm_mxfp8_tflops": round(flops / t8 / 1e9, 1),
            "gemm_speedup_mxfp4_over_mxfp8": round(t8 / t4, 3),
            "quantizer_shape": [r, c], "quant_mxfp4_ms": round(tq4, 4), "quant_mxfp8_ms": round(tq8, 4),
            "paper_context": "the paper reports almost 2x over FP8 for linear layers on an RTX 5090 (Section 1); "
                             "up to 2x forward and 1.5x backward (Section 5)"}


def recorded(config, name, key):
    """A figure measured offline with rocprofv3 counters (HBM bytes per GEMM launch scaled by a plain
    copy kernel of known size; shader clock while the GEMMs run), read from the committed summary
    profiles/<name>; None if it is not there."""
    path = os.path.join(ROOT, "profiles", name.format(config=config))
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def lower_bound_ms(layers):
    """Time no implementation of the path can beat on this chip's published peaks:
    6*T*I*O / peak MFMA + (bytes of the memory-bound steps) / 8 TB/s."""
    total = 0.0
    for l in layers:
        t, i, o = l.t, l.i, l.o
        mem = 2.65625 * (t * i + o * i)          # forward quantizers of X and W (codes, scales, mask)
        mem += 2.53125 * 2 * t * o               # backward quantizers of dy, row and transposed
        mem += 1.0625 * (o * i + t * i)          # re-quantization of W_q and X_q along the other dimension
        total += 6.0 * t * i * o / (PEAK_FP4_TFLOPS * 1e12) + mem / (PEAK_HBM_GBS * 1e9)
    return total * 1e3


def mfma_ceiling(q, torch, layer, cus, wall_khz):
    """What the bare matrix-core instruction sustains on this machine right now: the library's register-only loop of
    v_mfma_scale_f32_32x32x64_f8f6f4 (one block of 4 waves per compute unit) on the first 32 KiB of the first layer's
    quantized activations and 8 KiB of their scale bytes, timed by events on the current stream; the shader clock it
    held comes from the kernel's own clock counters."""
    codes = layer.xq_codes.reshape(-1)[:32768].contiguous()
    scales = layer.xq_scales.reshape(-1)[:8192].contiguous()
    sink = torch.empty((cus * 256,), dtype=torch.float32, device=codes.device)
    ctr = torch.zeros((2,), dtype=torch.int64, device=codes.device)
    warm, iters = 20000, 100000
    q.check(q.quartet_probe_mfma_ceiling(codes, scales, warm, cus, sink))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    q.check(q.quartet_probe_mfma_ceiling(codes, scales, iters, cus, sink, ctr))
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    c = ctr.cpu().tolist()
    flop = cus * 4.0 * iters * 16 * 2 * 32 * 32 * 64
    return {"TFLOPs": round(flop / ms / 1e9, 1), "ms": round(ms, 2), "blocks": cus, "iterations": iters,
            "clock_ghz": round(c[0] / c[1] * wall_khz / 1e6, 3) if c[1] > 0 and wall_khz > 0 else None,
            "what": "register-only loop of the GEMM's matrix-core instruction on this run's quantized activations: "
                    "no LDS, no memory traffic; the chip lowers its clock under it (power), so this, not 10.1 PFLOP/s, "
                    "is what the instruction alone reaches on this box"}


def time_config(q, torch, synth, config, steps, warmup, rounding):
    """Whole-path rate of another configuration: K timed steps, no event pairs, wall clock around a synchronize."""
    cfg = synth.CONFIGS[config]
    layers = [Layer(q, torch, synth.device_layer(config, li)) for li in range(len(cfg["layers"]))]
    ws_bytes = max(l.ws_bytes for l in layers)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda:0")
    for s in range(warmup):
        for l in layers:
            l.step(q, ws, s, rounding)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        for l in layers:
            l.step(q, ws, 1000 + s, rounding)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    flops = sum(l.flops for l in layers)
    return {"config": config, "workload": cfg["name"], "layers": len(layers), "steps": steps,
            "ms_per_step": round(dt * 1e3 / steps, 4), "value": round(flops * steps / dt / 1e12, 2), "unit": "TFLOP/s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    from paper_2505_14669_amd import binding as q
    from paper_2505_14669_amd import synth

    torch.cuda.set_device(0)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    wall_khz = q.quartet_wall_clock_khz()
    cfg = synth.CONFIGS[args.config]
    layers = [Layer(q, torch, synth.device_layer(args.config, li), args.hadamard_block) for li in range(len(cfg["layers"]))]
    ws_bytes = max(l.ws_bytes for l in layers)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    flops_step = sum(l.flops for l in layers)
    launches_per_step = 11 * len(layers)   # capacity (wider Hadamard blocks): 2 + 1 forward, (2 + 1) x 2 backward, + 2 epilogue kernels; blocks of 32 need 4

    def one_step(step):
        for l in layers:
            l.step(q, ws, step, args.rounding)

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()

    def read_profile(cap):
        kinds = (ctypes.c_int * cap)()
        ms = (ctypes.c_float * cap)()
        n = q.quartet_profile_read(kinds, ms, cap)
        if n < 0:
            q.check(n)
        q.quartet_profile_enable(0)
        per = {}
        for kk, m in zip(kinds[:n], ms[:n]):
            per.setdefault(q.KIND_NAMES[kk], []).append(m)
        return per

    # timed region: only the dominant kernel (the GEMM) carries event pairs, each costs a few microseconds of stream time;
    # its blocks also add their shader-clock and constant-clock ticks to two device counters (two atomics per block)
    clock_ctr = torch.zeros((2,), dtype=torch.int64, device="cuda:0")
    q.check(q.quartet_profile_clock(clock_ctr))
    q.check(q.quartet_profile_kinds(1 << q.QUARTET_KIND_GEMM))
    q.check(q.quartet_profile_enable(launches_per_step * args.steps))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(1000 + s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_kind = read_profile(launches_per_step * args.steps)
    q.check(q.quartet_profile_clock(None))
    clock_ticks = clock_ctr.cpu().tolist()

    # one more step, outside the timed region, with every launch bracketed: the per-kind time shares
    q.check(q.quartet_profile_kinds(0xFFFFFFFF))
    q.check(q.quartet_profile_enable(launches_per_step))
    t1 = time.perf_counter()
    one_step(2000)
    torch.cuda.synchronize()
    dt_all = time.perf_counter() - t1
    per_kind_all = read_profile(launches_per_step)

    gemm_ms = per_kind.get("gemm", [])
    gemm_flops_step = flops_step               # three GEMMs of 2*T*I*O each = 6*T*I*O
    gemm_total_ms = sum(gemm_ms)
    achieved = gemm_flops_step * args.steps / (gemm_total_ms * 1e-3) / 1e12 if gemm_total_ms > 0 else 0.0

    # per GEMM shape, from the same event pairs (launch order inside a step: forward, dW, dX of each layer): the rate,
    # and the share of the HBM peak that the minimum traffic (operands once, result once) comes to -- products with a
    # short inner dimension and an fp32 result are bound by the result's stores, not by the matrix cores
    # (Hadamard blocks up to 128: the backward pass runs its two products, dW and dX, in one launch: two records per layer)
    by_shape = {}
    per_layer = 2 if args.hadamard_block <= 128 else 3
    if len(gemm_ms) == per_layer * len(layers) * args.steps:
        for idx, m_s in enumerate(gemm_ms):
            l, which = layers[(idx // per_layer) % len(layers)], idx % per_layer
            fwd, dw, dx = (l.t, l.o, l.i), (l.o, l.i, l.t), (l.t, l.i, l.o)
            key = ((fwd,), (dw, dx))[which] if per_layer == 2 else ((fwd,), (dw,), (dx,))[which]
            by_shape.setdefault(key, []).append(m_s)
    gemm_by_shape = []
    for products, v in sorted(by_shape.items()):
        avg = sum(v) / len(v)
        flops = sum(2.0 * m * n * k for (m, n, k) in products)
        min_bytes = sum((m + n) * k * (0.5 + 1.0 / 32.0) + 4.0 * m * n for (m, n, k) in products)
        entry = {"m": products[0][0], "n": products[0][1], "k": products[0][2]}
        if len(products) == 2:
            entry = {"products": [list(pr) for pr in products], "what": "dW and dX of one layer in one launch"}
        entry.update({"launches": len(v), "avg_ms": round(avg, 4), "TFLOPs": round(flops / avg / 1e9, 1),
                      "frac_mfma": round(flops / avg / 1e9 / PEAK_FP4_TFLOPS, 4),
                      "min_GBps": round(min_bytes / avg / 1e6, 1),
                      "frac_hbm": round(min_bytes / avg / 1e6 / PEAK_HBM_GBS, 4)})
        gemm_by_shape.append(entry)

    ms_per_step = dt * 1e3 / args.steps
    big_gemm = any(((l.t + 255) // 256) * ((l.o + 255) // 256) >= 160 for l in layers)
    result = {
        "metric": "Quartet linear fwd+bwd TFLOP/s at 1 GPU; quantizer GB/s; % of MXFP4/HBM roofline",
        "value": round(flops_step / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 (E2M1 x E8M0/32) operands, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg['name']}, {len(layers)} linear layers fwd+bwd, "
                               f"backward rounding {'stochastic' if args.rounding == 0 else 'nearest'}"
                               + ("" if args.hadamard_block == 32 else f", Hadamard block {args.hadamard_block}"),
                   "layers": [[l.name, l.t, l.i, l.o] for l in layers]},
        "roofline": {"bound": "mfma",
                     "kernel": ("gemm_mxfp4_stream_kernel" if big_gemm else "gemm_mxfp4_stream_tile_kernel") + " (all three GEMMs of every layer: the forward product, and dW with dX in one launch)",
                     "achieved": round(achieved, 2), "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_FP4_TFLOPS, 4),
                     "traffic": recorded(args.config, "gemm_config{config}_hbm_traffic.txt", "traffic_bytes_per_launch"),
                     "traffic_source": "recorded, not measured in this run: rocprofv3 FETCH_SIZE / WRITE_SIZE per launch from "
                                       f"profiles/gemm_config{args.config}_hbm_traffic.txt",
                     "avg_launch_ms": round(gemm_total_ms / max(len(gemm_ms), 1), 4), "launches": len(gemm_ms),
                     "compute_units": cus},
        "gemm_by_shape": gemm_by_shape,
        "lower_bound_ms_per_step": round(lower_bound_ms(layers), 4),
        "kernel_time_share": {k: round(sum(v) / (dt_all * 1e3), 4) for k, v in sorted(per_kind_all.items())},
    }
    if clock_ticks[1] > 0 and wall_khz > 0:   # the shader clock the chip held under the GEMM kernel, measured by the kernel itself in the timed region
        clock = clock_ticks[0] / clock_ticks[1] * wall_khz / 1e6
        peak_obs = cus * clock * 1e9 * 16384 / 1e12
        result["roofline"].update(observed_clock_ghz=round(clock, 3), peak_at_observed_clock=round(peak_obs, 1),
                                  frac_at_observed_clock=round(achieved / peak_obs, 4),
                                  clock_source="measured in the timed region: shader-clock over constant-clock ticks summed "
                                               "over the blocks of every large-tile GEMM launch")
    if not args.no_ceiling and args.hadamard_block == 32:
        ceil = mfma_ceiling(q, torch, layers[0], cus, wall_khz)
        result["roofline"]["mfma_ceiling"] = ceil
        result["roofline"]["frac_of_ceiling"] = round(achieved / ceil["TFLOPs"], 4) if ceil["TFLOPs"] > 0 else None
    if args.breakdown:
        for k, v in sorted(per_kind_all.items()):
            print(f"  {k:10s} launches {len(v):4d} total {sum(v):9.3f} ms  ({sum(v) / (dt_all * 1e3) * 100:5.1f} % of one fully bracketed step)",
                  file=sys.stderr)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if args.fp8_compare:
        result["fp8_comparison"] = fp8_compare(q, torch, layers)
    first = layers[0] if args.hadamard_block == 32 else None     # the CPU baseline's sample comes from this layer's tensors
    del layers, ws
    torch.cuda.empty_cache()
    if not args.no_quant_sweep:
        result["quantizer_sweep"] = quant_sweep(q, torch, synth)
        torch.cuda.empty_cache()
    if not args.no_other_configs:
        result["other_configs"] = [time_config(q, torch, synth, c, 10, 3, args.rounding) for c in (1, 2, 3) if c != args.config]
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.config, first, q)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
