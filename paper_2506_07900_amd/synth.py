"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds NO arithmetic of the method (no pooling, scoring, selection or
attention): it only draws tensors.  It depends on numpy alone, so both the CPU
oracle's tests and the HIP path's tests can use it without importing each other.

All tensors are bf16, returned as numpy uint16 bit patterns (round-to-nearest-even
from float32 draws).  Layouts: q [l, Hq, d]; k, v [Hkv, l, d].

Recipe: numpy Generator(PCG64(seed)); Q, K, V ~ N(0,1).  "Planted" key blocks: per
key-value head, distinct block indices drawn uniformly from [1, nb-3]; every key
row of a planted block is sqrt(d)*u + 0.1*eps, where u is the unit vector along the
mean of all query rows of that head's group and eps ~ N(0, I).  Heavy-tailed
sequences multiply key row t by exp(z_t), z_t ~ N(0,1).
"""
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20250607


def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    x = np.ascontiguousarray(x, np.float32)
    u = x.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 array (exact)."""
    b = np.ascontiguousarray(b, np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Config:
    """One benchmark configuration (shapes follow the five stated workloads)."""
    name: str
    kind: str                 # "prefill" | "decode"
    seqlen: int               # prefill length, or cached context before the first decode step
    n_q_heads: int
    n_kv_heads: int
    topk: int
    n_planted: int
    batch: int = 1
    steps: int = 0            # decode steps
    head_dim: int = 128
    block_size: int = 64
    kernel_size: int = 32
    kernel_stride: int = 16
    n_init_blocks: int = 1
    n_local_blocks: int = 2
    seed: int = BASE_SEED
    ragged: bool = False      # decode: contexts drawn uniformly from [seqlen_min, seqlen]
    seqlen_min: int = 0
    heavy_tail_first: int = 0  # decode: number of leading sequences with lognormal key norms


CONFIGS = [
    Config("prefill_2k_g4", "prefill", 2048, 4, 1, 8, 4, seed=BASE_SEED + 0),
    Config("prefill_32k", "prefill", 32768, 32, 2, 16, 32, seed=BASE_SEED + 1),
    Config("prefill_128k", "prefill", 131072, 32, 2, 16, 128, seed=BASE_SEED + 2),
    Config("decode_128k", "decode", 131072, 32, 2, 16, 128, steps=1000, seed=BASE_SEED + 3),
    Config("decode_ragged_b8", "decode", 131072, 32, 2, 16, 32, batch=8, steps=200,
           seed=BASE_SEED + 4, ragged=True, seqlen_min=16384, heavy_tail_first=4),
]


def _normal_bf16(rng, shape, chunk_rows=1 << 15):
    """N(0,1) float32 draws rounded to bf16, generated in row chunks to bound memory."""
    out = np.empty(shape, np.uint16)
    flat = out.reshape(shape[0], -1)
    for a in range(0, shape[0], chunk_rows):
        b = min(shape[0], a + chunk_rows)
        flat[a:b] = f32_to_bf16_bits(rng.standard_normal((b - a, flat.shape[1]), dtype=np.float32))
    return out


def _group_mean_direction(q_bits, n_kv_heads):
    """Unit vector along the mean query row of each key-value head's group.  q [rows, Hq, d]."""
    rows, Hq, d = q_bits.shape
    G = Hq // n_kv_heads
    acc = np.zeros((Hq, d), np.float64)
    for a in range(0, rows, 1 << 14):
        acc += bf16_bits_to_f32(q_bits[a:a + (1 << 14)]).astype(np.float64).sum(axis=0)
    mean = acc.reshape(n_kv_heads, G, d).sum(axis=1) / float(rows * G)
    return mean / np.linalg.norm(mean, axis=1, keepdims=True)


def _plant_indices(rng, n_planted, n_blocks):
    """Sorted distinct planted block indices for one head, uniform over [1, n_blocks-3]."""
    hi = n_blocks - 3
    if n_planted <= 0 or hi < 1:
        return np.zeros((0,), np.int64)
    n = min(n_planted, hi)
    return np.sort(rng.choice(np.arange(1, hi + 1), size=n, replace=False))


@dataclass
class PrefillInputs:
    q: np.ndarray            # uint16 [l, Hq, d]
    k: np.ndarray            # uint16 [Hkv, l, d]
    v: np.ndarray            # uint16 [Hkv, l, d]
    planted: list = field(default_factory=list)   # per kv head: sorted block indices


def make_sequence(seed, seqlen, n_q_heads, n_kv_heads, head_dim=128, block_size=64,
                  n_planted=0, heavy_tail=False, n_q_rows=None):
    """One sequence: q [n_q_rows or seqlen, Hq, d], k/v [Hkv, seqlen, d], planted blocks.

    Draw order is fixed: Q, K, V, then per head (planted indices, planted noise), then the
    heavy-tail factors."""
    rng = np.random.Generator(np.random.PCG64(seed))
    d = head_dim
    nq = seqlen if n_q_rows is None else n_q_rows
    q = _normal_bf16(rng, (nq, n_q_heads, d))
    kf = rng.standard_normal((n_kv_heads, seqlen, d), dtype=np.float32)
    v = _normal_bf16(rng, (seqlen, n_kv_heads * d)).reshape(seqlen, n_kv_heads, d)
    v = np.ascontiguousarray(v.transpose(1, 0, 2))
    planted = []
    n_blocks = (seqlen + block_size - 1) // block_size
    if n_planted > 0:
        u = _group_mean_direction(q, n_kv_heads)
        for h in range(n_kv_heads):
            idx = _plant_indices(rng, n_planted, n_blocks)
            for j in idx:
                eps = rng.standard_normal((block_size, d), dtype=np.float32)
                kf[h, j * block_size:(j + 1) * block_size] = (
                    np.sqrt(np.float32(d)) * u[h].astype(np.float32)[None, :] + np.float32(0.1) * eps)
            planted.append(idx)
    else:
        planted = [np.zeros((0,), np.int64) for _ in range(n_kv_heads)]
    if heavy_tail:
        z = rng.standard_normal((n_kv_heads, seqlen, 1), dtype=np.float32)
        kf = kf * np.exp(z)
    k = f32_to_bf16_bits(kf)
    return PrefillInputs(q=q, k=k, v=v, planted=planted)


def make_prefill(cfg):
    """Inputs of a prefill config (batch 1)."""
    assert cfg.kind == "prefill"
    return make_sequence(cfg.seed, cfg.seqlen, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                         cfg.block_size, cfg.n_planted)


@dataclass
class DecodeInputs:
    seqlens0: np.ndarray     # int32 [B] cached context before the first step
    capacity: int            # cache rows per sequence (>= max seqlens0 + steps)
    k_cache: np.ndarray      # uint16 [B, Hkv, capacity, d]; rows >= seqlens0[b] are zero
    v_cache: np.ndarray
    q_steps: np.ndarray      # uint16 [steps, B, Hq, d]
    k_steps: np.ndarray      # uint16 [steps, B, Hkv, d]
    v_steps: np.ndarray
    planted: list = field(default_factory=list)   # [b][h] -> block indices


def make_decode(cfg, steps=None, seqlen=None, seqlen_min=None, batch=None):
    """Inputs of a decode config: an initial cache per sequence and per-step q, k, v rows.

    The planted direction of a sequence is taken from the mean of its own step queries."""
    assert cfg.kind == "decode"
    steps = cfg.steps if steps is None else steps
    L = cfg.seqlen if seqlen is None else seqlen
    Lmin = cfg.seqlen_min if seqlen_min is None else seqlen_min
    B = cfg.batch if batch is None else batch
    d, Hq, Hkv, m = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads, cfg.block_size
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    if cfg.ragged:
        seqlens0 = rng.integers(Lmin, L + 1, size=B).astype(np.int32)
    else:
        seqlens0 = np.full((B,), L, np.int32)
    capacity = int(-(-(int(seqlens0.max()) + steps) // 256) * 256)
    q_steps = _normal_bf16(rng, (steps, B * Hq * d)).reshape(steps, B, Hq, d)
    k_steps = _normal_bf16(rng, (steps, B * Hkv * d)).reshape(steps, B, Hkv, d)
    v_steps = _normal_bf16(rng, (steps, B * Hkv * d)).reshape(steps, B, Hkv, d)
    k_cache = np.zeros((B, Hkv, capacity, d), np.uint16)
    v_cache = np.zeros((B, Hkv, capacity, d), np.uint16)
    planted = []
    for b in range(B):
        Lb = int(seqlens0[b])
        n_pl = cfg.n_planted if not cfg.ragged else int(round(cfg.n_planted * Lb / 32768.0))
        seq = make_sequence(cfg.seed * 1000 + b, Lb, Hq, Hkv, d, m, n_planted=0,
                            heavy_tail=False, n_q_rows=1)
        # planted blocks and heavy tails are applied here so that u comes from the step queries
        sub = np.random.Generator(np.random.PCG64(cfg.seed * 1000 + 500 + b))
        kf = bf16_bits_to_f32(seq.k)
        u = _group_mean_direction(np.ascontiguousarray(q_steps[:, b]), Hkv) if steps > 0 else None
        pl = []
        n_blocks = (Lb + m - 1) // m
        for h in range(Hkv):
            idx = _plant_indices(sub, n_pl if u is not None else 0, n_blocks)
            for j in idx:
                eps = sub.standard_normal((m, d), dtype=np.float32)
                rows = slice(j * m, min((j + 1) * m, Lb))
                kf[h, rows] = (np.sqrt(np.float32(d)) * u[h].astype(np.float32)[None, :]
                               + np.float32(0.1) * eps)[: rows.stop - rows.start]
            pl.append(idx)
        if b < cfg.heavy_tail_first:
            z = sub.standard_normal((Hkv, Lb, 1), dtype=np.float32)
            kf = kf * np.exp(z)
        k_cache[b, :, :Lb] = f32_to_bf16_bits(kf)
        v_cache[b, :, :Lb] = seq.v
        planted.append(pl)
    return DecodeInputs(seqlens0=seqlens0, capacity=capacity, k_cache=k_cache, v_cache=v_cache,
                        q_steps=q_steps, k_steps=k_steps, v_steps=v_steps, planted=planted)
