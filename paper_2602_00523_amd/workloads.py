"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only draws random numbers and lays them out in the shapes of the
benchmark configurations; it contains none of the method's arithmetic (no
entropy, no tree rule, no attention, no acceptance).  numpy only.

Stand-ins: the paper evaluates on image/video question-answering and captioning
sets with trained 72B/7B model pairs (Sec. 5.1); neither data nor weights are
available, so Q/K/V and logits are i.i.d. Gaussians at the same shapes
(64 query heads, 8 KV heads, head_dim 128, vocabulary 152064, KV lengths of a
few thousand image tokens up to video length).
"""
from __future__ import annotations

import numpy as np

MAX_NODES = 64
SEED_BASE = 523000

# name -> shape/params.  Tree parameters of c2/c4/c5 are the paper's (Sec. 5.1
# implementation details); toy and c3 widen/narrow them as the configuration
# text asks (depth up to 10, width 1..16 for c3).
CONFIGS = {
    "toy": dict(index=0, dtype="f32", Hq=4, Hkv=1, d=64, kv_len=256, vocab=1024, B=1, layers=1, steps=32,
                tree=dict(d_min=2, d_max=6, w_min=1, w_max=6, k=8, n_max=16)),
    "c2": dict(index=1, dtype="bf16", Hq=64, Hkv=8, d=128, kv_len=4096, vocab=152064, B=1, layers=1, steps=32,
               tree=dict(d_min=3, d_max=8, w_min=2, w_max=10, k=10, n_max=64)),
    "c3": dict(index=2, dtype="bf16", Hq=64, Hkv=8, d=128, kv_len=16384, vocab=152064, B=1, layers=1, steps=256,
               tree=dict(d_min=3, d_max=10, w_min=1, w_max=16, k=16, n_max=64)),
    "c4": dict(index=3, dtype="bf16", Hq=64, Hkv=8, d=128, kv_len=(2048, 12288), vocab=152064, B=8, layers=1,
               steps=16, tree=dict(d_min=3, d_max=8, w_min=2, w_max=10, k=10, n_max=64)),
    "c5": dict(index=4, dtype="bf16", Hq=64, Hkv=8, d=128, kv_len=32768, vocab=152064, B=1, layers=80, steps=8,
               tree=dict(d_min=3, d_max=8, w_min=2, w_max=10, k=10, n_max=64)),
}


def seed_for(config: str, step: int = 0, stream: int = 0) -> int:
    return SEED_BASE + 1000 * CONFIGS[config]["index"] + step + 100003 * stream


def rng(seed: int) -> np.random.Generator:
    return np.random.default_rng(seed)


# ---- storage-type helpers (bit manipulation only) -------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs and +-inf)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array -> the config's storage type: float32 as is, bf16 as uint16 bits."""
    x = np.ascontiguousarray(x, np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


# ---- draws ------------------------------------------------------------------

def gaussian(seed: int, shape, dtype: str, scale: float = 1.0) -> np.ndarray:
    z = rng(seed).standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        z *= np.float32(scale)
    return to_storage(z, dtype)


def attention_inputs(seed: int, B: int, Hq: int, Hkv: int, d: int, kv_lens, dtype: str, pad_tokens: int = 0):
    """Q [B,64,Hq,d], Kt/Vt [B,64,Hkv,d] and one packed cache [sum(kv_lens)+pad, Hkv, d] for K and for V, N(0,1).

    Returns a dict with kv_start (token offsets of each sequence in the packed
    cache), kv_len, and the element strides of the cache.
    """
    kv_lens = np.asarray(kv_lens, np.int32).reshape(B)
    kv_start = np.zeros(B, np.int64)
    kv_start[1:] = np.cumsum(kv_lens.astype(np.int64))[:-1]
    total = int(kv_lens.sum()) + pad_tokens
    g = rng(seed)

    def draw(shape):
        return to_storage(g.standard_normal(shape, dtype=np.float32), dtype)

    return dict(
        Q=draw((B, MAX_NODES, Hq, d)), Kt=draw((B, MAX_NODES, Hkv, d)), Vt=draw((B, MAX_NODES, Hkv, d)),
        Kc=draw((max(total, 1), Hkv, d)), Vc=draw((max(total, 1), Hkv, d)),
        kv_start=kv_start, kv_len=kv_lens, kv_token_stride=Hkv * d, kv_head_stride=d)


def ragged_kv_lens(seed: int, B: int, lo: int, hi: int) -> np.ndarray:
    return rng(seed).integers(lo, hi + 1, size=B).astype(np.int32)


# Mean full-vocabulary entropy (nats) of softmax(beta * z), z ~ N(0,1)^152064 stored as bf16, over six seeds, as
# printed by tests/golden/make_entropy_scale_table.py; used only to steer the logit scale toward a requested entropy.
# Individual rows scatter around it (the low end depends on the gap between the two largest draws), which is fine:
# the table shapes inputs, the kernels report what the entropy actually is.
_ENTROPY_TO_SCALE_152064 = [
    (11.81, 0.5), (11.43, 1.0), (10.81, 1.5), (9.94, 2.0), (8.83, 2.5), (7.56, 3.0), (6.91, 3.25), (6.28, 3.5),
    (5.70, 3.75), (5.19, 4.0), (4.71, 4.25), (4.30, 4.5), (3.94, 4.75), (3.61, 5.0), (3.10, 5.5), (2.67, 6.0),
    (2.37, 6.5), (2.09, 7.0), (1.69, 8.0), (1.41, 9.0), (1.19, 10.0), (0.89, 12.0), (0.70, 14.0), (0.48, 17.0),
    (0.37, 20.0), (0.24, 25.0), (0.19, 30.0), (0.13, 60.0),
]


def scale_for_entropy(h: float) -> float:
    """Logit scale beta that steers Gaussian logits over the 152064-token vocabulary toward entropy h (nats)."""
    hs = np.array([e for e, _ in _ENTROPY_TO_SCALE_152064][::-1])
    bs = np.array([b for _, b in _ENTROPY_TO_SCALE_152064][::-1])
    return float(np.interp(h, hs, bs))


def ar1_entropy_targets(seed: int, steps: int, lo: float = 0.0, hi: float = 6.0, phi: float = 0.8,
                        mean: float = 3.0, sigma: float = 1.0) -> np.ndarray:
    """Seeded AR(1) sequence of target entropies clipped to [lo, hi] (the paper reports entropy to be
    strongly autocorrelated over decoding steps without printing coefficients; phi = 0.8 is a choice)."""
    g = rng(seed)
    h = np.empty(steps)
    cur = mean
    for t in range(steps):
        h[t] = cur
        cur = float(np.clip(mean + phi * (cur - mean) + sigma * g.standard_normal(), lo, hi))
    return h


def entropy_targets(config: str, steps: int) -> np.ndarray:
    """Per-step target entropies of a 72B-shape configuration (c3: AR(1) in [0,6]; others: uniform in [0.05,5])."""
    if config == "c3":
        return ar1_entropy_targets(seed_for(config, 0, 7), steps)
    return rng(seed_for(config, 0, 7)).uniform(0.05, 5.0, size=steps)


def toy_temperatures(steps: int) -> np.ndarray:
    return rng(seed_for("toy", 0, 7)).uniform(0.1, 3.0, size=steps)


def draft_logits(seed: int, rows: int, vocab: int, dtype: str, scale: float) -> np.ndarray:
    """[rows, vocab] Gaussian logits times `scale` in the storage type."""
    return gaussian(seed, (rows, vocab), dtype, scale)


def target_logits_from_draft(seed: int, draft_row_f32: np.ndarray, rows: int, dtype: str, noise: float) -> np.ndarray:
    """Per-node target logits = the step's draft row plus seeded Gaussian noise of std `noise` (so confident
    steps accept deep paths and uncertain steps reject early)."""
    g = rng(seed)
    out = np.empty((rows, draft_row_f32.shape[0]), np.float32)
    for r in range(rows):
        out[r] = draft_row_f32 + np.float32(noise) * g.standard_normal(draft_row_f32.shape[0], dtype=np.float32)
    return to_storage(out, dtype)
