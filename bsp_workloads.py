"""Seeded synthetic inputs for the block-structured-pruning path.

This module only draws random tensors of the shapes, dtypes and value distributions of the
BERT-base / BERT-large linear layers that the paper prunes (Sec. 4.2: L=12, H=768 for the
base models; the large shape is H=1024, FFN 4096, 24 layers).  It holds none of the
method's arithmetic (no norms, thresholds, packing or products), so both the CPU oracle's
tests and the GPU tests may use it.  GLUE-fine-tuned checkpoints are not available; iid
Gaussian weights with std 0.02 (the BERT initialiser range) stand in for them.

All tensors are returned as host numpy float32 arrays.  For a low-precision dtype the
values are first rounded to that dtype (library conversion, round-to-nearest-even), so the
float32 array holds exactly the bits both sides will see.
"""
from __future__ import annotations

import numpy as np
import torch

PAPER_SEED = 42  # the paper's default seed (Sec. 5.4)

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def to_dtype_values(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array whose values are exactly representable in `dtype`."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    return torch.from_numpy(a).to(_TORCH_DT[dtype]).to(torch.float32).numpy()


def normal(seed, shape, std, dtype="f32") -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed))
    a = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return to_dtype_values(a, dtype)


def random_keep_mask(seed, B, N, k) -> np.ndarray:
    """uint8 [B, N]; in every row exactly k seeded uniform-random positions are 1."""
    rng = np.random.Generator(np.random.Philox(seed))
    keep = np.zeros((B, N), dtype=np.uint8)
    for b in range(B):
        keep[b, rng.permutation(N)[:k]] = 1
    return keep


def bernoulli_keep_mask(seed, B, N, p) -> np.ndarray:
    """uint8 [B, N]; every position kept independently with probability p (ragged k_b)."""
    rng = np.random.Generator(np.random.Philox(seed))
    return (rng.random((B, N)) < p).astype(np.uint8)


def layer(seed, T, M, N, dtype, bias=True):
    """One linear layer's tensors: X [T,N] ~ N(0,1), W [M,N] ~ N(0,0.02), bias [M] ~ N(0,0.02)."""
    d = dict(T=T, M=M, N=N, dtype=dtype,
             X=normal(seed * 1000 + 1, (T, N), 1.0, dtype),
             W=normal(seed * 1000 + 2, (M, N), 0.02, dtype))
    d["bias"] = normal(seed * 1000 + 3, (M,), 0.02, dtype) if bias else None
    return d


def skewed_weight(seed, M, N, R, dtype="f32", sigma=1.0):
    """Stress input: N(0,0.02) weights times log-normal per-column and per-row-block scales,
    so some columns survive in most blocks and the kept count per block is skewed."""
    rng = np.random.Generator(np.random.Philox(seed))
    W = rng.standard_normal(size=(M, N), dtype=np.float32) * np.float32(0.02)
    col = np.exp(sigma * rng.standard_normal(N)).astype(np.float32)
    blk = np.exp(sigma * rng.standard_normal(M // R)).astype(np.float32)
    W = W * col[None, :] * np.repeat(blk, R)[:, None]
    return to_dtype_values(W, dtype)


def n_keep_for_rate(n_groups: int, num: int, den: int) -> int:
    """Groups kept for a compression rate num/den: floor(n*den/num), so rate >= requested."""
    return (n_groups * den) // num


# ----------------------------------------------------------------------------------------
# The five workloads.  seed = 42 + index.  `tokens` lets tests shrink the token count; the
# weight shapes are always the real ones unless `shrink` divides them.
# ----------------------------------------------------------------------------------------
def config1(tokens=128):
    """BERT-base attention projection, fp32, R=16, exactly half the columns kept per block."""
    d = layer(PAPER_SEED + 1, tokens, 768, 768, "f32")
    d.update(R=16, keep=random_keep_mask((PAPER_SEED + 1) * 1000 + 4, 768 // 16, 768, 384))
    return d


def config2(tokens=4096):
    """BERT-base FFN up-projection, bf16, R=16, top third of groups per row-block (3x)."""
    d = layer(PAPER_SEED + 2, tokens, 3072, 768, "bf16")
    d.update(R=16, n_keep=256, scope="block")
    return d


BASE_SHAPES = [("qkv", 2304, 768), ("attn_out", 768, 768), ("ffn_up", 3072, 768), ("ffn_down", 768, 3072)]
LARGE_SHAPES = [("qkv", 3072, 1024), ("attn_out", 1024, 1024), ("ffn_up", 4096, 1024), ("ffn_down", 1024, 4096)]
RATES = [(3, 2), (2, 1), (3, 1), (5, 1)]


def config3(tokens=8192):
    """BERT-base encoder-layer linear set, bf16, R=16, per-matrix rate drawn from RATES."""
    rng = np.random.Generator(np.random.Philox(PAPER_SEED + 3))
    out = []
    for i, (name, M, N) in enumerate(BASE_SHAPES):
        d = layer((PAPER_SEED + 3) * 10 + i, tokens, M, N, "bf16")
        num, den = RATES[int(rng.integers(len(RATES)))]
        d.update(name=name, R=16, rate=(num, den), scope="matrix",
                 n_keep=n_keep_for_rate((M // 16) * N, num, den))
        out.append(d)
    return out


def config4(tokens=8192, R=16, shapes=None):
    """BERT-large / RoBERTa-large linear set, bf16, 5x compression, matrix-scope percentile."""
    out = []
    for i, (name, M, N) in enumerate(shapes or LARGE_SHAPES):
        d = layer((PAPER_SEED + 4) * 10 + i, tokens, M, N, "bf16")
        d.update(name=name, R=R, rate=(5, 1), scope="matrix", n_keep=n_keep_for_rate((M // R) * N, 5, 1))
        out.append(d)
    return out


def config5_shapes(layers=24):
    """(M, N) of every matrix of a BERT-large weight set (per layer Q, K, V, O, up, down), in buffer order:
    the matrices of width 1024 of all layers first, then the down-projections (width 4096), as a flat
    parameter buffer that groups tensors of one shape would hold them."""
    narrow = ([(1024, 1024)] * 4 + [(4096, 1024)]) * layers
    wide = [(1024, 4096)] * layers
    return narrow + wide


def config5(layers=24):
    """fp32 weight set laid end to end in one buffer plus (offset, M, N) descriptors."""
    shapes = config5_shapes(layers)
    total = sum(m * n for m, n in shapes)
    rng = np.random.Generator(np.random.Philox(PAPER_SEED + 5))
    buf = rng.standard_normal(size=total, dtype=np.float32)
    buf *= np.float32(0.02)
    desc, off = [], 0
    for m, n in shapes:
        desc.append((off, m, n))
        off += m * n
    return dict(W=buf, desc=desc, R=16, eps=1e-6, lam=1e-4, rate=(5, 1))
