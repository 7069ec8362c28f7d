"""ctypes wrapper around the C oracle (`infllmv2_oracle.c`).

TEST INFRASTRUCTURE ONLY.  Marshals numpy arrays to the C functions, which hold the arithmetic
of the method.  The one exception is select_blocks_shared, the query-block-shared comparison
variant (not the report's method): it averages the per-token block scores the C oracle returns
over each query block and ranks them here, in plain Python loops.  bf16 tensors are numpy uint16
arrays of bit patterns.  One sequence per call.

Layouts (C-contiguous):
  q      [Tq, Hq, d]    row t is the query token at position pos[t]
  k, v   [Hkv, l, d]
  ck     [Hkv, n_c, d]
  block_idx [Hkv, Tq, topk] int32, ascending, -1 padded
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "infllmv2_oracle.c")
# INFLLMV2_ORACLE_SANITIZE=undefined: a second build with UndefinedBehaviorSanitizer (any report aborts),
# so that the pins can be run once more over instrumented code (tests/test_sanitizers.py)
_SANITIZE = os.environ.get("INFLLMV2_ORACLE_SANITIZE", "")
_LIB = os.path.join(_HERE, "libinfllmv2_oracle%s.so" % ("_" + _SANITIZE if _SANITIZE else ""))
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (CPU only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        san = ["-g", "-fsanitize=" + _SANITIZE, "-fno-sanitize-recover=all"] if _SANITIZE else []
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off"] + san + ["-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, f64, vp = ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.oracle_num_kernels.restype = i32
        lib.oracle_num_kernels.argtypes = [i32, i32, i32]
        lib.oracle_compress_keys.restype = i32
        lib.oracle_compress_keys.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
        lib.oracle_kernel_scores.restype = None
        lib.oracle_kernel_scores.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, f64, vp]
        lib.oracle_select_blocks.restype = None
        lib.oracle_select_blocks.argtypes = [vp, vp, vp] + [i32] * 11 + [f64, vp, vp, vp, i32]
        lib.oracle_num_coarse.restype = i32
        lib.oracle_num_coarse.argtypes = [i32, i32]
        lib.oracle_coarse_kernels.restype = i32
        lib.oracle_coarse_kernels.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        lib.oracle_kernel_scores_coarse.restype = None
        lib.oracle_kernel_scores_coarse.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [f64, vp, vp]
        lib.oracle_select_blocks_coarse.restype = None
        lib.oracle_select_blocks_coarse.argtypes = [vp, vp, vp, vp] + [i32] * 13 + [f64, vp, vp, vp, i32]
        lib.oracle_sparse_attn.restype = None
        lib.oracle_sparse_attn.argtypes = [vp, vp, vp, vp, vp] + [i32] * 7 + [f64, vp, vp, vp]
        lib.oracle_sparse_attn_bwd.restype = None
        lib.oracle_sparse_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp] + [i32] * 7 + [f64, vp, vp, vp, vp, vp, vp]
        lib.oracle_sparse_attn_tree.restype = None
        lib.oracle_sparse_attn_tree.argtypes = [vp, vp, vp, vp, vp] + [i32] * 8 + [f64, vp, vp]
        lib.oracle_f64_to_bf16.restype = ctypes.c_uint16
        lib.oracle_f64_to_bf16.argtypes = [f64]
        lib.oracle_bf16_to_f64.restype = f64
        lib.oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
        _lib = lib
    return _lib


@dataclass
class Params:
    """Hyper-parameters of section 2.1 (names follow the paper: m, p, s, k)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    block_size: int = 64        # m
    kernel_size: int = 32       # p
    kernel_stride: int = 16     # s
    topk: int = 16              # k, total blocks per query including the forced ones
    n_init_blocks: int = 1
    n_local_blocks: int = 2
    softmax_scale: float = None
    lse_coarse_ratio: int = 1   # rho = s_c / s of the approximate log-sum-exp; 1 = exact

    def __post_init__(self):
        if self.softmax_scale is None:
            self.softmax_scale = float(self.head_dim) ** -0.5


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_kernels(l, p, s):
    return int(_load().oracle_num_kernels(int(l), int(p), int(s)))


def f64_to_bf16(x):
    return int(_load().oracle_f64_to_bf16(float(x)))


def bf16_to_f64(b):
    return float(_load().oracle_bf16_to_f64(int(b)))


def compress_keys(k, prm):
    """k uint16 [Hkv, l, d] -> (ck_f64 [Hkv, n_c, d], ck_bf16 uint16 [Hkv, n_c, d])."""
    lib = _load()
    k = _u16(k)
    Hkv, l, d = k.shape
    n_c = num_kernels(l, prm.kernel_size, prm.kernel_stride)
    ck64 = np.zeros((Hkv, n_c, d), np.float64)
    ckb = np.zeros((Hkv, n_c, d), np.uint16)
    got = lib.oracle_compress_keys(_ptr(k), Hkv, l, d, prm.kernel_size, prm.kernel_stride,
                                   _ptr(ck64), _ptr(ckb))
    assert got == n_c
    return ck64, ckb


def num_coarse(n, rho):
    return int(_load().oracle_num_coarse(int(n), int(rho)))


def coarse_kernels(ck, rho):
    """ck uint16 [Hkv, n_c, d] -> (ckc_f64, ckc_bf16 uint16) [Hkv, n_cc, d]."""
    lib = _load()
    ck = _u16(ck)
    Hkv, n_c, d = ck.shape
    n_cc = num_coarse(n_c, rho)
    c64 = np.zeros((Hkv, n_cc, d), np.float64)
    cb = np.zeros((Hkv, n_cc, d), np.uint16)
    got = lib.oracle_coarse_kernels(_ptr(ck), Hkv, n_c, d, int(rho), _ptr(c64), _ptr(cb))
    assert got == n_cc
    return c64, cb


def kernel_scores(q, ck, pos, prm, want_lse=False, coarse_path=None):
    """Group-mean kernel scores r [Hkv, Tq, n_c] (0 beyond the visible kernels); with
    prm.lse_coarse_ratio > 1 the approximate log-sum-exp is used (want_lse: also return it,
    [Hkv, Tq, G]).  coarse_path=True takes the approximate-LSE code path even for ratio 1 (where it
    must reproduce the exact scores)."""
    lib = _load()
    q = _u16(q)
    ck = _u16(ck)
    pos = np.ascontiguousarray(pos, np.int32)
    Tq, Hq, d = q.shape
    Hkv, n_c, _ = ck.shape
    assert Hq == prm.n_q_heads and Hkv == prm.n_kv_heads and pos.shape == (Tq,)
    r = np.zeros((Hkv, Tq, n_c), np.float64)
    if prm.lse_coarse_ratio > 1 if coarse_path is None else coarse_path:
        _, ckc = coarse_kernels(ck, prm.lse_coarse_ratio)
        lse = np.zeros((Hkv, Tq, Hq // Hkv), np.float64)
        lib.oracle_kernel_scores_coarse(_ptr(q), _ptr(ck), _ptr(ckc), _ptr(pos), Tq, Hq, Hkv, d, n_c,
                                        ckc.shape[1], prm.kernel_size, prm.kernel_stride,
                                        prm.lse_coarse_ratio, float(prm.softmax_scale), _ptr(r), _ptr(lse))
        return (r, lse) if want_lse else r
    assert not want_lse
    lib.oracle_kernel_scores(_ptr(q), _ptr(ck), _ptr(pos), Tq, Hq, Hkv, d, n_c,
                             prm.kernel_size, prm.kernel_stride, float(prm.softmax_scale), _ptr(r))
    return r


def select_blocks(q, ck, pos, prm, want_scores=False, coarse_path=None):
    """-> block_idx int32 [Hkv, Tq, topk], margins fp64 [Hkv, Tq, 2] (, R [Hkv, Tq, nb])."""
    lib = _load()
    q = _u16(q)
    ck = _u16(ck)
    pos = np.ascontiguousarray(pos, np.int32)
    Tq, Hq, d = q.shape
    Hkv, n_c, _ = ck.shape
    assert Hq == prm.n_q_heads and Hkv == prm.n_kv_heads and pos.shape == (Tq,)
    idx = np.full((Hkv, Tq, prm.topk), -1, np.int32)
    margins = np.zeros((Hkv, Tq, 2), np.float64)
    nb_cap = int(pos.max()) // prm.block_size + 1 if Tq else 1
    R = np.zeros((Hkv, Tq, nb_cap), np.float64) if want_scores else None
    if prm.lse_coarse_ratio > 1 if coarse_path is None else coarse_path:
        _, ckc = coarse_kernels(ck, prm.lse_coarse_ratio)
        lib.oracle_select_blocks_coarse(_ptr(q), _ptr(ck), _ptr(ckc), _ptr(pos), Tq, Hq, Hkv, d, n_c,
                                        ckc.shape[1], prm.block_size, prm.kernel_size, prm.kernel_stride,
                                        prm.topk, prm.n_init_blocks, prm.n_local_blocks,
                                        prm.lse_coarse_ratio, float(prm.softmax_scale),
                                        _ptr(idx), _ptr(margins), _ptr(R), nb_cap)
    else:
        lib.oracle_select_blocks(_ptr(q), _ptr(ck), _ptr(pos), Tq, Hq, Hkv, d, n_c,
                                 prm.block_size, prm.kernel_size, prm.kernel_stride, prm.topk,
                                 prm.n_init_blocks, prm.n_local_blocks, float(prm.softmax_scale),
                                 _ptr(idx), _ptr(margins), _ptr(R), nb_cap)
    return (idx, margins, R) if want_scores else (idx, margins)


def sparse_attn(q, k, v, pos, block_idx, prm, want_probs_sum=False):
    """-> out fp64 [Tq, Hq, d], lse fp64 [Tq, Hq] (, probs_sum [Tq, Hq])."""
    lib = _load()
    q = _u16(q)
    k = _u16(k)
    v = _u16(v)
    pos = np.ascontiguousarray(pos, np.int32)
    block_idx = np.ascontiguousarray(block_idx, np.int32)
    Tq, Hq, d = q.shape
    Hkv, l, _ = k.shape
    assert v.shape == k.shape and pos.shape == (Tq,)
    topk = block_idx.shape[-1]
    assert block_idx.shape == (Hkv, Tq, topk)
    out = np.zeros((Tq, Hq, d), np.float64)
    lse = np.zeros((Tq, Hq), np.float64)
    ps = np.zeros((Tq, Hq), np.float64) if want_probs_sum else None
    lib.oracle_sparse_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(pos), _ptr(block_idx), Tq, Hq, Hkv, d,
                           l, prm.block_size, topk, float(prm.softmax_scale),
                           _ptr(out), _ptr(lse), _ptr(ps))
    return (out, lse, ps) if want_probs_sum else (out, lse)


def sparse_attn_tree(q, k, v, block_idx, tree_mask, l_ctx, prm):
    """Tree-style draft verification: q uint16 [n, Hq, d] are the n <= 64 drafted tokens at cache
    positions l_ctx .. l_ctx+n-1, tree_mask uint64 [n] (bit j of word t: query t attends draft j),
    block_idx int32 [Hkv, n, topk] -> out fp64 [n, Hq, d], lse fp64 [n, Hq]."""
    lib = _load()
    q = _u16(q)
    k = _u16(k)
    v = _u16(v)
    block_idx = np.ascontiguousarray(block_idx, np.int32)
    tree_mask = np.ascontiguousarray(tree_mask, np.uint64)
    n, Hq, d = q.shape
    Hkv, l, _ = k.shape
    topk = block_idx.shape[-1]
    assert v.shape == k.shape and block_idx.shape == (Hkv, n, topk) and tree_mask.shape == (n,) and n <= 64
    out = np.zeros((n, Hq, d), np.float64)
    lse = np.zeros((n, Hq), np.float64)
    lib.oracle_sparse_attn_tree(_ptr(q), _ptr(k), _ptr(v), _ptr(block_idx), _ptr(tree_mask), n, int(l_ctx),
                                Hq, Hkv, d, l, prm.block_size, topk, float(prm.softmax_scale),
                                _ptr(out), _ptr(lse))
    return out, lse


def sparse_attn_bwd(q, k, v, dout, pos, block_idx, prm, want_mag=False):
    """Gradients of sparse_attn's output for the upstream gradient dout (uint16 bf16 bits [Tq, Hq, d]),
    block sets fixed -> dq fp64 [Tq, Hq, d], dk, dv fp64 [Hkv, l, d]; with want_mag also the three
    arrays of term magnitudes (the scale of a rounding-error tolerance)."""
    lib = _load()
    q, k, v, dout = _u16(q), _u16(k), _u16(v), _u16(dout)
    pos = np.ascontiguousarray(pos, np.int32)
    block_idx = np.ascontiguousarray(block_idx, np.int32)
    Tq, Hq, d = q.shape
    Hkv, l, _ = k.shape
    topk = block_idx.shape[-1]
    assert dout.shape == q.shape and v.shape == k.shape and block_idx.shape == (Hkv, Tq, topk)
    dq = np.zeros((Tq, Hq, d), np.float64)
    dk = np.zeros((Hkv, l, d), np.float64)
    dv = np.zeros((Hkv, l, d), np.float64)
    mags = [np.zeros_like(dq), np.zeros_like(dk), np.zeros_like(dv)] if want_mag else [None] * 3
    lib.oracle_sparse_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(pos), _ptr(block_idx), Tq, Hq, Hkv, d,
                               l, prm.block_size, topk, float(prm.softmax_scale), _ptr(dq), _ptr(dk), _ptr(dv),
                               *[_ptr(x) if x is not None else None for x in mags])
    return (dq, dk, dv, *mags) if want_mag else (dq, dk, dv)


def select_blocks_shared(q, ck, prm, want_scores=False, qblocks=None):
    """Query-block-shared selection -- NOT the report's method (section 2.1.3 argues for token-level
    queries); a comparison variant in which the m tokens of a query block attend one common block set.
    Query block I (tokens m*I .. m*I+m-1 of a sequence of l = len(q) tokens) scores key-value block j by
    the mean over its tokens of their per-token block relevance (Eq. 1 of section 2.1.2, as computed by
    select_blocks); the first n_init blocks and the last n_local blocks up to I are forced, and the
    min(topk, I+1) best are taken, ties to the lower index.  All candidates n_init <= j <= I - n_local
    are wholly visible to every token of the query block.
    -> block_idx int32 [Hkv, n_qb, topk] ascending, padded with -1, margins fp64 [Hkv, n_qb, 2]
       (score of the last pick, best score not picked; nan if none) (, Rq fp64 [Hkv, n_qb, nb]).
    With qblocks (a list of query-block indices) only those rows are computed; the others stay -1."""
    q = _u16(q)
    l = q.shape[0]
    m = prm.block_size
    Hkv = prm.n_kv_heads
    n_qb = (l + m - 1) // m
    which = list(range(n_qb)) if qblocks is None else [int(I) for I in qblocks]
    pos = np.concatenate([np.arange(I * m, min((I + 1) * m, l), dtype=np.int32) for I in which]) if which \
        else np.zeros((0,), np.int32)
    _, _, Rt = select_blocks(np.ascontiguousarray(q[pos]), ck, pos, prm, want_scores=True)
    row_of = {int(t): a for a, t in enumerate(pos)}
    idx = np.full((Hkv, n_qb, prm.topk), -1, np.int32)
    margins = np.full((Hkv, n_qb, 2), np.nan)
    Rq = np.full((Hkv, n_qb, n_qb), -np.inf)
    for h in range(Hkv):
        R = {t: Rt[h, a] for t, a in row_of.items()}
        for I in which:
            toks = range(I * m, min((I + 1) * m, l))
            n_init = min(prm.n_init_blocks, I + 1)
            lo_local = max(n_init, I - prm.n_local_blocks + 1)
            forced = list(range(n_init)) + list(range(lo_local, I + 1))
            cand = list(range(n_init, lo_local))
            score = {}
            for j in cand:
                total = 0.0
                for t in toks:
                    total += R[t][j]
                score[j] = total / len(toks)
                Rq[h, I, j] = score[j]
            for j in forced:
                Rq[h, I, j] = np.inf
            n_pick = min(prm.topk, I + 1) - len(forced)
            order = sorted(cand, key=lambda j: (-score[j], j))
            picks = order[:n_pick]
            if picks:
                margins[h, I, 0] = score[picks[-1]]
            if len(order) > n_pick and n_pick >= 0:
                margins[h, I, 1] = score[order[n_pick]]
            sel = sorted(forced + picks)
            idx[h, I, :len(sel)] = sel
    return (idx, margins, Rq) if want_scores else (idx, margins)
