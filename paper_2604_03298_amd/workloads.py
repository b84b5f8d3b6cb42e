"""Seeded synthetic weight tensors (bf16; fp16 and fp32 variants) for the tests and the benchmark.

This module only makes inputs.  It holds none of the codec's arithmetic and is
the one module that both the CPU oracle's tests and the GPU path's tests use, so
that both sides always see the same bytes.  Tensors are returned as numpy arrays of
bit patterns: uint16 for bf16 and fp16, uint32 for fp32.

The tensors stand in for the HuggingFace checkpoints the paper measures on
(Table II), which are not available offline: shapes follow 7B-70B decoder layers,
values follow the near-Gaussian per-tensor statistics of Sec. III (Obs. 3 and 5).
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def gaussian(n_elems: int, std: float, seed: int) -> np.ndarray:
    """i.i.d. N(0, std^2) drawn in float64, rounded to float32 and then to bf16."""
    g = _rng(seed)
    out = np.empty(n_elems, dtype=np.uint16)
    step = 1 << 22
    for s in range(0, n_elems, step):
        e = min(n_elems, s + step)
        out[s:e] = f32_to_bf16_bits((std * g.standard_normal(e - s)).astype(np.float32))
    return out


def gaussian_fp16(n_elems: int, std: float, seed: int) -> np.ndarray:
    """i.i.d. N(0, std^2) drawn in float64, rounded to IEEE half; uint16 bit patterns."""
    return (std * _rng(seed).standard_normal(n_elems)).astype(np.float16).view(np.uint16)


def gaussian_fp32(n_elems: int, std: float, seed: int) -> np.ndarray:
    """i.i.d. N(0, std^2) drawn in float64, rounded to float32; uint32 bit patterns."""
    return (std * _rng(seed).standard_normal(n_elems)).astype(np.float32).view(np.uint32)


def config1(seed: int = 1, rows: int = 1024, cols: int = 4096) -> np.ndarray:
    """Single matrix, i.i.d. N(0, 0.02^2)."""
    return gaussian(rows * cols, 0.02, seed)


def layer_matrix(rows: int, cols: int, seed: int) -> np.ndarray:
    """One projection matrix of the 7B-style layer: each row ~ N(0, s^2) with s log-uniform
    in [0.005, 0.05]; each entry with probability 0.001 replaced by an outlier of
    magnitude 20 s and random sign."""
    g = _rng(seed)
    s = np.exp(g.uniform(np.log(0.005), np.log(0.05), size=rows))
    out = np.empty(rows * cols, dtype=np.uint16)
    rstep = max(1, (1 << 22) // cols)
    for r0 in range(0, rows, rstep):
        r1 = min(rows, r0 + rstep)
        sr = s[r0:r1, None]
        v = g.standard_normal((r1 - r0, cols)) * sr
        hit = g.random((r1 - r0, cols)) < 0.001
        sign = np.where(g.random((r1 - r0, cols)) < 0.5, -1.0, 1.0)
        v = np.where(hit, 20.0 * sr * sign, v)
        out[r0 * cols:r1 * cols] = f32_to_bf16_bits(v.astype(np.float32)).reshape(-1)
    return out


def norm_vector(n: int, seed: int) -> np.ndarray:
    g = _rng(seed)
    return f32_to_bf16_bits((1.0 + 0.05 * g.standard_normal(n)).astype(np.float32))


def config2_spec(hidden: int = 4096, ffn: int = 11008):
    """(name, rows, cols, seed) of the nine tensors of the 7B-style decoder layer."""
    return [
        ("q_proj", hidden, hidden, 20), ("k_proj", hidden, hidden, 21),
        ("v_proj", hidden, hidden, 22), ("o_proj", hidden, hidden, 23),
        ("gate_proj", hidden, ffn, 24), ("up_proj", hidden, ffn, 25),
        ("down_proj", ffn, hidden, 26),
        ("input_norm", 1, hidden, 27), ("post_norm", 1, hidden, 28),
    ]


def config2(hidden: int = 4096, ffn: int = 11008):
    """Yields (name, uint16 array) for the 7B-style layer (full size by default)."""
    for name, rows, cols, seed in config2_spec(hidden, ffn):
        if rows == 1:
            yield name, norm_vector(cols, seed)
        else:
            yield name, layer_matrix(rows, cols, seed)


def config3(n_blocks: int = 4096, block: int = 16384, seed: int = 3):
    """Edge-case mix: each data block is all-zero, one repeated value, Student-t (df=3,
    scale 0.02) or uniform random 16-bit patterns (NaN/Inf/denormals included).
    Returns (tensor, category per block)."""
    g = _rng(seed)
    cat = g.permutation(n_blocks) % 4
    out = np.zeros(n_blocks * block, dtype=np.uint16)
    for i in range(n_blocks):
        sl = slice(i * block, (i + 1) * block)
        c = cat[i]
        if c == 1:
            out[sl] = f32_to_bf16_bits(np.float32(0.02 * g.standard_normal()).reshape(1))[0]
        elif c == 2:
            out[sl] = f32_to_bf16_bits((0.02 * g.standard_t(3, size=block)).astype(np.float32))
        elif c == 3:
            out[sl] = g.integers(0, 1 << 16, size=block, dtype=np.uint16)
    return out, cat


def config3_by_category(n_blocks: int = 4096, block: int = 16384, seed: int = 3):
    """The same blocks gathered into four tensors, one per category (0 zero, 1 constant,
    2 heavy-tailed, 3 random bits)."""
    t, cat = config3(n_blocks, block, seed)
    t = t.reshape(n_blocks, block)
    return [np.ascontiguousarray(t[cat == c]).reshape(-1) for c in range(4)]


def config4_std(index: int, seed: int = 4) -> float:
    """Per-tensor std of the large-layer stream, log-uniform in [0.003, 0.03]."""
    g = _rng(seed)
    return float(np.exp(g.uniform(np.log(0.003), np.log(0.03), size=32))[index])


def config4_tensor(index: int, rows: int = 8192, cols: int = 28672, seed: int = 4) -> np.ndarray:
    return gaussian(rows * cols, config4_std(index, seed), 400 + index)


def config5_spec(n_layers: int = 8, hidden: int = 8192, ffn: int = 28672):
    """(rows, cols, seed) of the offload scenario's tensors, all N(0, 0.015^2)."""
    spec = []
    for i in range(n_layers):
        spec.append((hidden, hidden, 500 + 2 * i))
        spec.append((hidden, ffn, 501 + 2 * i))
    return spec


def gpu_gaussian(torch, rows, cols, std, seed, dtype=None):
    """N(0, std^2) drawn on the GPU, as bit patterns: int16 for bf16 (default) and float16, int32 for float32."""
    dtype = torch.bfloat16 if dtype is None else dtype
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.empty(rows * cols, dtype=dtype, device="cuda")
    step = 1 << 25      # float64 draws: float32 samplers emit exact zeros, which would force n = 8
    for s in range(0, x.numel(), step):
        e = min(x.numel(), s + step)
        x[s:e] = (torch.randn(e - s, generator=g, device="cuda", dtype=torch.float64) * std).to(dtype)
    return x.view(torch.int32 if dtype == torch.float32 else torch.int16)


def config4_device(torch, index: int, rows: int = 8192, cols: int = 28672):
    """Tensor `index` (0..31) of the large-layer stream drawn on the GPU (15 GB of numpy normals take
    minutes): N(0, config4_std(index)^2), seed 4000 + index.  The host sees the same bytes through a
    device-to-host copy."""
    return gpu_gaussian(torch, rows, cols, config4_std(index), 4000 + index)


def config5_device(torch, index: int, spec=None):
    """Tensor `index` (0..15) of the offload scenario drawn on the GPU: N(0, 0.015^2), seeds of config5_spec."""
    rows, cols, seed = (spec or config5_spec())[index]
    return gpu_gaussian(torch, rows, cols, 0.015, seed)
