"""Seeded synthetic inputs for the checksum-protected GEMM.

This module serves both the CPU oracle and the HIP library with the SAME bits
and holds none of the method's arithmetic: no GEMM, no checksum, no flag logic.
It only draws numbers, rounds fp32 draws once to the storage type, and lists
the ViT-shaped workloads.

The paper measures on DeiT/ViT layers fed with ImageNet-1k (Sec. IV-A); neither
the weights nor the dataset are available, so tensors of the same *shapes* with
prescribed value distributions stand in for them:
  int8   : uniform integers in [-128, 127]
  bf16/fp16 activations ~ N(0, 1), weights ~ N(0, 0.02)
  attention probabilities: row-wise softmax of N(0, 1) logits
Bit flips follow the paper's fault model (Sec. II-A "Formulation to Quantify
Resilience", Sec. III-A): one flip per run in a layer output; any bit for
integers, an exponent or a mantissa bit for floating point.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20231003

DTYPES = ("i8", "bf16", "f16")


def seed_for(config: int, tensor_index: int) -> int:
    """Fixed seed table: one seed per (config, tensor) pair."""
    return BASE_SEED + 100 * int(config) + int(tensor_index)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


# ----------------------------------------------------------------------------
# storage-type conversion of fp32 draws (input preparation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to IEEE half (nearest even, numpy's conversion) and return uint16 bits."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def to_storage_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f16":
        return f32_to_f16_bits(x)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
def gen_int8(shape, seed: int) -> np.ndarray:
    """Uniform integers in [-128, 127] as int8."""
    return _rng(seed).integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)


def gen_normal_bits(shape, seed: int, std: float, dtype: str) -> np.ndarray:
    """N(0, std^2) drawn in fp32, rounded once to bf16/fp16; returns uint16 bits."""
    x = _rng(seed).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return to_storage_bits(x, dtype)


def gen_softmax_bits(shape, seed: int, dtype: str) -> np.ndarray:
    """Row-wise softmax (fp32) of N(0,1) logits, rounded to the storage type.

    Stands in for the attention-probability operand of the attn x V product."""
    z = _rng(seed).standard_normal(size=shape, dtype=np.float32)
    z = z - z.max(axis=-1, keepdims=True)
    p = np.exp(z)
    p = p / p.sum(axis=-1, keepdims=True)
    return to_storage_bits(p.astype(np.float32), dtype)


def gen_operands(dtype: str, M: int, N: int, K: int, seed_a: int, seed_b: int,
                 trans_b: bool = True, batch: int = 1, a_kind: str = "act",
                 b_kind: str = "weight"):
    """A (batch, M, K) and B stored as (batch, N, K) when trans_b else (batch, K, N).

    int8 -> int8 arrays; bf16/f16 -> uint16 bit patterns.
    a_kind/b_kind in {"act" (std 1), "weight" (std 0.02), "softmax"}."""
    bshape = (batch, N, K) if trans_b else (batch, K, N)
    ashape = (batch, M, K)
    if dtype == "i8":
        return gen_int8(ashape, seed_a), gen_int8(bshape, seed_b)

    def one(shape, seed, kind):
        if kind == "softmax":
            return gen_softmax_bits(shape, seed, dtype)
        return gen_normal_bits(shape, seed, 1.0 if kind == "act" else 0.02, dtype)

    return one(ashape, seed_a, a_kind), one(bshape, seed_b, b_kind)


# ----------------------------------------------------------------------------
# single-bit flips in the stored output C
# ----------------------------------------------------------------------------
def gen_flips(n: int, M: int, N: int, dtype: str, seed: int, batch: int = 1) -> np.ndarray:
    """n seeded flips, each a row (batch_index, row, col, bit) of an int64 array.

    i8 path (C is int32): bit uniform in 0..31.
    f16: with probability 1/2 an exponent bit (10..14) else a mantissa bit (0..9).
    bf16: exponent bits 7..14, mantissa bits 0..6. The sign bit is never flipped
    for floating point (the fault model names exponent and mantissa bits)."""
    g = _rng(seed)
    pos = g.integers(0, batch * M * N, size=n, dtype=np.int64)
    if dtype == "i8":
        bit = g.integers(0, 32, size=n, dtype=np.int64)
    else:
        man_hi, exp_lo, exp_hi = (9, 10, 14) if dtype == "f16" else (6, 7, 14)
        is_exp = g.integers(0, 2, size=n, dtype=np.int64).astype(bool)
        ebit = g.integers(exp_lo, exp_hi + 1, size=n, dtype=np.int64)
        mbit = g.integers(0, man_hi + 1, size=n, dtype=np.int64)
        bit = np.where(is_exp, ebit, mbit)
    out = np.empty((n, 4), dtype=np.int64)
    out[:, 0] = pos // (M * N)
    out[:, 1] = (pos % (M * N)) // N
    out[:, 2] = pos % N
    out[:, 3] = bit
    return out


# ----------------------------------------------------------------------------
# workloads (shapes of ViT-B/16 at 224^2 and ViT-L/16 at 384^2)
# ----------------------------------------------------------------------------
def vit_block_gemms(tokens: int, hidden: int, heads: int, mlp: int, batch: int):
    """The six GEMM classes of one transformer block as dicts.

    Linear layers multiply by the transposed weight (weight stored N x K);
    Q.K^T also has its second operand stored N x K; attn.V has it stored K x N."""
    hd = hidden // heads
    Mtok = batch * tokens
    return [
        dict(name="qkv", M=Mtok, N=3 * hidden, K=hidden, batch=1, trans_b=True, a_kind="act", b_kind="weight"),
        dict(name="qk", M=tokens, N=tokens, K=hd, batch=batch * heads, trans_b=True, a_kind="act", b_kind="act"),
        dict(name="av", M=tokens, N=hd, K=tokens, batch=batch * heads, trans_b=False, a_kind="softmax", b_kind="act"),
        dict(name="proj", M=Mtok, N=hidden, K=hidden, batch=1, trans_b=True, a_kind="act", b_kind="weight"),
        dict(name="fc1", M=Mtok, N=mlp, K=hidden, batch=1, trans_b=True, a_kind="act", b_kind="weight"),
        dict(name="fc2", M=Mtok, N=hidden, K=mlp, batch=1, trans_b=True, a_kind="act", b_kind="weight"),
    ]


CONFIGS = {
    # 0: single int8 GEMM, ViT-B attention projection shape, 1000 flips
    0: dict(dtype="i8", gemms=[dict(name="proj_b1", M=197, N=768, K=768, batch=1, trans_b=True,
                                    a_kind="act", b_kind="weight")], flips=1000),
    # 1: bf16 ViT-B MLP fc1 at batch 64 (the benchmark workload)
    1: dict(dtype="bf16", gemms=[dict(name="fc1_b64", M=12608, N=3072, K=768, batch=1, trans_b=True,
                                      a_kind="act", b_kind="weight")], flips=0),
    # 2: full ViT-B/16 block, bf16, batch 32
    2: dict(dtype="bf16", gemms=vit_block_gemms(197, 768, 12, 3072, 32), blocks=12, flips=0),
    # 3: ViT-L/16 at 384^2, int8, batch 64
    3: dict(dtype="i8", gemms=vit_block_gemms(577, 1024, 16, 4096, 64), blocks=24, flips=0),
    # 4: injection campaign on ViT-B fc2 (int8 and fp16)
    4: dict(dtype="i8", gemms=[dict(name="fc2_b32", M=6304, N=768, K=3072, batch=1, trans_b=True,
                                    a_kind="act", b_kind="weight")], flips=100000, also="f16"),
}
