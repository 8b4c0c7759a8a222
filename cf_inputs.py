"""Seeded synthetic inputs for the decode block (shared by tests, smoke and bench).

This module holds no arithmetic of the method: it only names the Llama-shaped
configurations and draws tensors with the stated shapes and distributions.
Both the CPU oracle's tests and the HIP path's tests feed on the same arrays.

Recipe: one numpy PCG64 generator per (seed); draw order x, W_qkv, W_o,
k_cache, v_cache; every tensor is drawn in float32 and rounded to fp16 with
round-to-nearest-even.  x ~ N(0,1); weights ~ N(0, std 0.02); cached K/V rows
[0, L) ~ N(0,1); rows >= L are fp16 NaN when `poison` is set (correctness
runs: nothing may read them) and zero otherwise (timing runs).  The cache
capacity max_seq is L + 9 rows (default_max_seq below says why).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class BlockShape:
    name: str
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    kv_len: int          # default number of cached tokens L (== pos of the new token)
    batch: int = 1

    @property
    def n_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim


SHAPES = {
    "tiny": BlockShape("tiny", 512, 8, 8, 64, 10000.0, 256),
    "llama2_7b": BlockShape("llama2_7b", 4096, 32, 32, 128, 10000.0, 4096),
    "llama3_8b": BlockShape("llama3_8b", 4096, 32, 8, 128, 500000.0, 8192),
    "llama2_70b": BlockShape("llama2_70b", 8192, 64, 8, 128, 10000.0, 32768),
    # MHA blocks with more heads (d_model = 128 * heads), for the sweep of the team size against the head count
    # (the experiment with varying cluster sizes and head counts of the paper's evaluation section)
    "mha_64h": BlockShape("mha_64h", 8192, 64, 64, 128, 10000.0, 4096),
    "mha_128h": BlockShape("mha_128h", 16384, 128, 128, 128, 10000.0, 4096),
}


def default_max_seq(kv_len: int) -> int:
    """Capacity of a KV-cache head slice: the new token and eight spare rows.

    The byte stride between heads (max_seq * head_dim * 2) decides how the concurrent K/V streams of different
    heads spread over the memory channels.  Measured on MI355X with the 7B shape: capacities of kv_len + 128
    rows at KV 16384 and kv_len + 256 rows at KV 32768 (strides of the form 2^k + 2^(k-7) bytes) cost 10-15 %;
    kv_len + 1 ... + 64 rows are good at every length tried."""
    return kv_len + 9


def make_inputs(shape: BlockShape, seed: int, batch: int | None = None, kv_len: int | None = None,
                max_seq: int | None = None, poison: bool = True) -> dict:
    """Draw one layer's inputs as fp16 numpy arrays (host memory)."""
    B = shape.batch if batch is None else int(batch)
    L = shape.kv_len if kv_len is None else int(kv_len)
    S = default_max_seq(L) if max_seq is None else int(max_seq)
    assert 0 <= L < S
    rng = np.random.Generator(np.random.PCG64(seed))

    def normal(shp, std):
        a = rng.standard_normal(size=shp, dtype=np.float32)
        if std != 1.0:
            a *= np.float32(std)
        return a.astype(np.float16)

    D, nq, nkv, d = shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = normal((B, D), 1.0)
    w_qkv = normal((D, shape.n_qkv), 0.02)
    w_o = normal((nq * d, D), 0.02)
    fill = np.float16(np.nan) if poison else np.float16(0.0)
    k_cache = np.full((B, nkv, S, d), fill, dtype=np.float16)
    v_cache = np.full((B, nkv, S, d), fill, dtype=np.float16)
    if L > 0:
        k_cache[:, :, :L, :] = normal((B, nkv, L, d), 1.0)
        v_cache[:, :, :L, :] = normal((B, nkv, L, d), 1.0)
    return {"x": x, "w_qkv": w_qkv, "w_o": w_o, "k_cache": k_cache, "v_cache": v_cache,
            "pos": L, "batch": B, "max_seq": S, "shape": shape}


# ---------------------------------------------------------------------------------------------------
# Multi-Head Latent Attention block (weight-absorbed form), DeepSeek-V2-Lite-shaped
# ---------------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class MlaShape:
    name: str
    d_model: int
    n_heads: int
    nope_dim: int
    rope_dim: int
    kv_lora_rank: int
    v_head_dim: int
    rope_base: float
    kv_len: int
    batch: int = 1


MLA_SHAPES = {
    # the model the paper measures its fused MLA block on (hidden 2048, 16 heads, 128 + 64 query dimensions,
    # latent rank 512, value dimension 128); sequence length as in the paper's sweeps
    "deepseek_v2_lite": MlaShape("deepseek_v2_lite", 2048, 16, 128, 64, 512, 128, 10000.0, 4096),
}


def make_mla_inputs(shape: MlaShape, seed: int, batch: int | None = None, kv_len: int | None = None,
                    poison: bool = True) -> dict:
    """Seeded fp16 inputs of one MLA layer: unit-variance activations and cached rows, weights scaled by
    1/sqrt(fan-in) so that every intermediate stays of order one."""
    B = shape.batch if batch is None else int(batch)
    Lk = shape.kv_len if kv_len is None else int(kv_len)
    S = default_max_seq(Lk)
    rng = np.random.Generator(np.random.PCG64(seed))

    def normal(shp, std):
        return (rng.standard_normal(size=shp, dtype=np.float32) * np.float32(std)).astype(np.float16)

    D, nh, n, r, l, v = shape.d_model, shape.n_heads, shape.nope_dim, shape.rope_dim, shape.kv_lora_rank, shape.v_head_dim
    cache = np.full((B, S, l + r), np.float16(np.nan) if poison else np.float16(0.0), dtype=np.float16)
    if Lk > 0:
        cache[:, :Lk] = normal((B, Lk, l + r), 1.0)
    return {"x": normal((B, D), 1.0), "w_q": normal((D, nh * (n + r)), D ** -0.5), "w_kv": normal((D, l + r), D ** -0.5),
            "w_up": normal((nh, n, l), n ** -0.5), "w_down": normal((nh, l, v), l ** -0.5),
            "w_o": normal((nh * v, D), (nh * v) ** -0.5), "kv_cache": cache, "pos": Lk, "batch": B, "max_seq": S,
            "shape": shape}


# ---------------------------------------------------------------------------------------------------
# Feed-forward block (three weight matrices), Llama-shaped
# ---------------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class FfnShape:
    name: str
    d_model: int
    d_ff: int
    batch: int = 1


FFN_SHAPES = {
    "tiny": FfnShape("tiny", 512, 1376),
    "llama2_7b": FfnShape("llama2_7b", 4096, 11008),
    "llama3_8b": FfnShape("llama3_8b", 4096, 14336),
    "llama2_70b": FfnShape("llama2_70b", 8192, 28672),
}


def make_ffn_inputs(shape: FfnShape, seed: int, batch: int | None = None) -> dict:
    """Seeded fp16 inputs of one feed-forward block: z ~ N(0,1), the three matrices [d_ff, d_model] ~ N(0, std 0.02),
    drawn in the order z, W1, W2, W3 (fp32, rounded to fp16)."""
    B = shape.batch if batch is None else int(batch)
    rng = np.random.Generator(np.random.PCG64(seed))

    def normal(shp, std):
        return (rng.standard_normal(size=shp, dtype=np.float32) * np.float32(std)).astype(np.float16)

    D, F = shape.d_model, shape.d_ff
    return {"z": normal((B, D), 1.0), "w1": normal((F, D), 0.02), "w2": normal((F, D), 0.02), "w3": normal((F, D), 0.02),
            "batch": B, "shape": shape}
