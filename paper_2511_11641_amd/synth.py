"""Seeded synthetic inputs shaped like the layers the paper trains.

This module only draws random tensors and rounds them to the storage dtype.  It holds
none of the method's arithmetic (no norms, scores, selections or contractions), so that
both the CPU oracle's tests and the GPU path's tests can be fed from it.

Generator: numpy's Philox (counter based), keyed by ``(seed, stream)`` where ``stream``
is a small fixed integer per tensor, so every tensor is reproducible on its own.

Shapes follow the models of the paper's Tables 1 and 3 (GPT-2-Medium: d=1024, 16 heads
of 64, d_ff=4096, GELU; LLaMA-1B: d=2048, 32 heads of 64, SwiGLU d_ff=5461, RoPE).
Weights are N(0, 0.02^2) (GPT-2 style initialisation, the paper's from-scratch setting),
activations and upstream gradients N(0, 1).  ``structure="pretrained"`` rescales every
inner dimension of both members of a pair by independent log-normal factors, which gives
the wide spread of pair norms of a trained model (the paper's fine-tuning setting);
``structure="ties"`` duplicates inner dimensions so that exact score ties occur.
"""
from __future__ import annotations

import numpy as np

# fixed stream ids, one per tensor
_STREAMS = {
    "x": 1, "dy": 2,
    "wq": 10, "wk": 11, "wv": 12, "wo": 13, "bq": 14, "bk": 15, "bv": 16, "bo": 17,
    "w1": 20, "w1b": 21, "w2": 22, "b1": 23, "b2": 24,
    "scale1": 30, "scale2": 31, "dup": 32, "misc": 40,
}


def rng(seed: int, stream: str | int) -> np.random.Generator:
    s = _STREAMS[stream] if isinstance(stream, str) else int(stream)
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, s]))


def normal(seed: int, stream, shape, std: float = 1.0) -> np.ndarray:
    """float32 N(0, std^2) tensor."""
    return (rng(seed, stream).standard_normal(size=shape, dtype=np.float32) * np.float32(std))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 tensor to the storage dtype and return it as float32 values."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_bits(x))
    raise ValueError(dtype)


def _structure(seed, w1_rows, w2_cols, n_inner, structure):
    """Apply the value structure along the shared inner dimension.

    w1_rows: list of arrays whose axis 0 is the inner dimension (rows are a_j).
    w2_cols: list of arrays whose axis 1 is the inner dimension (columns are b_j).
    """
    if structure == "scratch":
        return
    if structure == "pretrained":
        s1 = np.exp(rng(seed, "scale1").standard_normal(n_inner) * 0.5).astype(np.float32)
        s2 = np.exp(rng(seed, "scale2").standard_normal(n_inner) * 0.5).astype(np.float32)
        for w in w1_rows:
            w *= s1[:, None]
        for w in w2_cols:
            w *= s2[None, :]
        return
    if structure == "ties":
        # every inner dimension in the second half of a run of 8 copies one of the first half
        src = np.arange(n_inner)
        blk = (src // 8) * 8
        off = src % 8
        src = np.where(off >= 4, blk + (off - 4), src)
        src = np.minimum(src, n_inner - 1)
        for w in w1_rows:
            w[:] = w[src]
        for w in w2_cols:
            w[:] = w[:, src]
        return
    raise ValueError(structure)


def ffn_layer(seed: int, T: int, d: int, n: int, *, gated: bool = False, dtype: str = "f32",
              structure: str = "scratch", bias: bool = True) -> dict:
    """One FFN coupled pair: X[T,d], W_1[n,d] (and W_up[n,d] when gated), W_2[d,n], dY[T,d].

    Storage is the Linear-layer layout ``W[out_features, in_features]``, ``y = x W^T``.
    """
    t = {
        "x": normal(seed, "x", (T, d)),
        "dy": normal(seed, "dy", (T, d)),
        "w1": normal(seed, "w1", (n, d), 0.02),
        "w2": normal(seed, "w2", (d, n), 0.02),
    }
    rows = [t["w1"]]
    if gated:
        t["w1b"] = normal(seed, "w1b", (n, d), 0.02)
        rows.append(t["w1b"])
    _structure(seed, rows, [t["w2"]], n, structure)
    if bias:
        t["b1"] = normal(seed, "b1", (n,), 0.02)
        t["b2"] = normal(seed, "b2", (d,), 0.02)
    return {k: round_to(v, dtype) for k, v in t.items()}


def attn_layer(seed: int, B: int, L: int, d: int, h: int, d_h: int, *, dtype: str = "f32",
               structure: str = "scratch", bias: bool = True) -> dict:
    """One attention block: X[B*L,d], W_q/W_k/W_v[h*d_h,d], W_o[d,h*d_h], dY[B*L,d]."""
    T = B * L
    n = h * d_h
    t = {
        "x": normal(seed, "x", (T, d)),
        "dy": normal(seed, "dy", (T, d)),
        "wq": normal(seed, "wq", (n, d), 0.02),
        "wk": normal(seed, "wk", (n, d), 0.02),
        "wv": normal(seed, "wv", (n, d), 0.02),
        "wo": normal(seed, "wo", (d, n), 0.02),
    }
    if structure == "pretrained":
        s = [np.exp(rng(seed, 50 + i).standard_normal(n) * 0.5).astype(np.float32) for i in range(4)]
        t["wq"] *= s[0][:, None]
        t["wk"] *= s[1][:, None]
        t["wv"] *= s[2][:, None]
        t["wo"] *= s[3][None, :]
    elif structure == "ties":
        _structure(seed, [t["wq"], t["wk"], t["wv"]], [t["wo"]], n, "ties")
    elif structure != "scratch":
        raise ValueError(structure)
    if bias:
        for nm, sz in (("bq", n), ("bk", n), ("bv", n), ("bo", d)):
            t[nm] = normal(seed, nm, (sz,), 0.02)
    return {k: round_to(v, dtype) for k, v in t.items()}


def keep_count(n: int, num: int, den: int) -> int:
    """Number of kept inner dimensions for a keep ratio num/den, in integer arithmetic."""
    return (n * num) // den


# The workloads named by the benchmark description, as keyword sets for the two makers.
CONFIGS = {
    # single FFN coupled pair, fp32, seed 0
    "c1_ffn_f32": dict(kind="ffn", seed=0, T=512, d=256, n=1024, gated=False, dtype="f32", act="gelu"),
    # GPT-2-Medium-shaped layer, bf16
    "c2_gpt2m_layer": dict(kind="layer", seed=1, B=8, L=1024, d=1024, h=16, d_h=64, d_ff=4096,
                           gated=False, dtype="bf16", act="gelu", rope=False, bias=True),
    # LLaMA-1B-shaped layer, bf16
    "c3_llama1b_layer": dict(kind="layer", seed=2, B=16, L=256, d=2048, h=32, d_h=64, d_ff=5461,
                             gated=True, dtype="bf16", act="swiglu", rope=True, bias=False),
    # LLaMA-7B-shaped layer (the paper's second pre-training model: 32 heads of 128 dims), bf16; not one of the metric's
    # configurations - the shape whose dense form and keep ratios above 1/2 need the 128-wide attention kernels
    "llama7b_layer": dict(kind="layer", seed=3, B=4, L=512, d=4096, h=32, d_h=128, d_ff=11008,
                          gated=True, dtype="bf16", act="swiglu", rope=True, bias=False),
}
