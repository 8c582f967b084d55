"""Seeded synthetic inputs for the Quartet linear-layer path.

Holds none of the method's arithmetic: only random tensors with the shapes and value
distributions of the paper's workloads (Llama-shaped linear layers with heavy-tailed
activations, outlier channels, small-variance weights and gradients; Section 5 "Speedup
results" uses Llama layer shapes at batch 64 x sequence 512), cast to bf16.  The tensors stand
in for activations of models trained on C4, which are not available and not needed.

bf16 tensors are numpy uint16 arrays of bit patterns.  The same module feeds the CPU oracle
(in tests) and the HIP path, so both see identical bytes.
"""
import numpy as np

# (name, tokens, in_features, out_features) of every linear layer in a configuration
CONFIGS = {
    1: dict(name="single linear 256x512x512",
            layers=[("linear", 256, 512, 512)]),
    2: dict(name="attention projections T=4096 d=2048",
            layers=[(n, 4096, 2048, 2048) for n in ("q", "k", "v", "o")]),
    3: dict(name="MLP T=8192 d=2048 ff=5632",
            layers=[("gate", 8192, 2048, 5632), ("up", 8192, 2048, 5632), ("down", 8192, 5632, 2048)]),
    4: dict(name="7B-shaped block T=16384 d=4096 ff=11008",
            layers=[(n, 16384, 4096, 4096) for n in ("q", "k", "v", "o")]
            + [("gate", 16384, 4096, 11008), ("up", 16384, 4096, 11008), ("down", 16384, 11008, 4096)]),
}

# quantizer-only sweep (configuration 5): bf16 matrices rows x cols
QUANT_SWEEP = [(16384, 4096), (16384, 11008), (16384, 14336)]


def f32_to_bf16(a):
    """Round-to-nearest-even cast of an fp32 array to bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(config, tensor_id, layer):
    return np.random.Generator(np.random.PCG64(1000 * config + tensor_id + 10 * layer))


def activations(config, layer, tokens, features):
    """X [tokens, features] fp32 before the bf16 cast."""
    g = _rng(config, 0, layer)
    if config == 1:
        x = g.standard_normal((tokens, features), dtype=np.float32)
        n_out = int(np.ceil(0.01 * features))
        cols = g.choice(features, size=n_out, replace=False)
        x[:, cols] *= np.float32(20.0)
        return x
    x = g.standard_t(3.0, size=(tokens, features)).astype(np.float32)
    rms = np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
    x /= rms
    if config >= 3:
        ch = np.exp(g.standard_normal(features)).astype(np.float32)
        x *= ch[None, :]
    return x


def weights(config, layer, out_features, in_features):
    g = _rng(config, 1, layer)
    return (g.standard_normal((out_features, in_features), dtype=np.float32) * np.float32(0.02))


def out_grads(config, layer, tokens, out_features):
    g = _rng(config, 2, layer)
    return (g.standard_normal((tokens, out_features), dtype=np.float32) * np.float32(1e-3))


def make_layer(config, layer):
    """bf16 X [T,I], W [O,I], dY [T,O] of one layer of configuration 1..4."""
    name, t, i, o = CONFIGS[config]["layers"][layer]
    return dict(name=name, tokens=t, in_features=i, out_features=o,
                x=f32_to_bf16(activations(config, layer, t, i)),
                w=f32_to_bf16(weights(config, layer, o, i)),
                dy=f32_to_bf16(out_grads(config, layer, t, o)))


def quant_sweep_matrix(index, rows=None, cols=None):
    """Configuration 5: N(0,1) with 0.1 % of the elements (random positions) scaled by 50."""
    r, c = QUANT_SWEEP[index]
    rows = r if rows is None else rows
    cols = c if cols is None else cols
    g = _rng(5, 0, index)
    x = g.standard_normal((rows, cols), dtype=np.float32)
    hit = g.random((rows, cols), dtype=np.float32) < np.float32(0.001)
    x[hit] *= np.float32(50.0)
    return f32_to_bf16(x)


def small_matrix(seed, rows, cols, kind="normal", scale=1.0):
    """Small test matrices (bf16) for parity cases: 'normal', 'outliers' (1 % columns x20),
    'heavy' (Student-t, nu=3), 'tiny' (N(0,1) * 2^-40), 'zeros'."""
    g = np.random.Generator(np.random.PCG64(seed))
    if kind == "zeros":
        return np.zeros((rows, cols), dtype=np.uint16)
    if kind == "heavy":
        x = g.standard_t(3.0, size=(rows, cols)).astype(np.float32)
    else:
        x = g.standard_normal((rows, cols), dtype=np.float32)
    if kind == "outliers":
        cols_hit = g.choice(cols, size=max(1, cols // 100), replace=False)
        x[:, cols_hit] *= np.float32(20.0)
    if kind == "tiny":
        x *= np.float32(2.0 ** -40)
    return f32_to_bf16(x * np.float32(scale))


# ------------------------------------------------------------------ device-side generation
# The same recipes drawn with torch's seeded generator on the GPU, for full-size benchmark tensors
# (hundreds of MiB each) that would take tens of seconds to draw on the host.  Different bytes than
# the numpy versions above, same shapes and distributions.

def _torch_gen(device, config, tensor_id, layer):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(1000 * config + tensor_id + 10 * layer)
    return g


def device_layer(config, layer, device="cuda:0"):
    """bf16 torch tensors X [T,I], W [O,I], dY [T,O] of one layer of configuration 1..4."""
    import torch
    name, t, i, o = CONFIGS[config]["layers"][layer]
    g = _torch_gen(device, config, 0, layer)
    if config == 1:
        x = torch.randn((t, i), generator=g, device=device)
        cols = torch.randperm(i, generator=g, device=device)[: -(-i // 100)]
        x[:, cols] *= 20.0
    else:
        # Student-t(3) = N(0,1) / sqrt(chi2(3)/3)
        z = torch.randn((t, i), generator=g, device=device)
        chi = torch.zeros((t, i), device=device)
        for _ in range(3):
            chi += torch.randn((t, i), generator=g, device=device) ** 2
        x = z / torch.sqrt(chi / 3.0)
        del z, chi
        x /= torch.sqrt(torch.mean(x * x, dim=1, keepdim=True))
        if config >= 3:
            x *= torch.exp(torch.randn((i,), generator=g, device=device))[None, :]
    w = torch.randn((o, i), generator=_torch_gen(device, config, 1, layer), device=device) * 0.02
    dy = torch.randn((t, o), generator=_torch_gen(device, config, 2, layer), device=device) * 1e-3
    return dict(name=name, tokens=t, in_features=i, out_features=o,
                x=x.to(torch.bfloat16).contiguous(), w=w.to(torch.bfloat16).contiguous(),
                dy=dy.to(torch.bfloat16).contiguous())


def device_quant_sweep_matrix(index, device="cuda:0"):
    import torch
    r, c = QUANT_SWEEP[index]
    g = _torch_gen(device, 5, 0, index)
    x = torch.randn((r, c), generator=g, device=device)
    hit = torch.rand((r, c), generator=g, device=device) < 0.001
    x = torch.where(hit, x * 50.0, x)
    return x.to(torch.bfloat16).contiguous()
