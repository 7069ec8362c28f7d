"""Thin Python binding over the C ABI declared in include/infllmv2.h.

Argument marshalling only: every function here has the name of the C entry point it calls
(minus the `infllmv2_` prefix), turns torch tensors into pointers + element strides, and
passes the current torch stream.  torch is used for device memory and streams, nothing else.
A missing library is an error: there is no fallback path.

Tensor layouts (bf16, CUDA/HIP device, head_dim contiguous):
  caches k, v, ck   [B, Hkv, T, d]
  queries, outputs  [B, T, Hq, d]   (decode: T = 1; draft verification: T = n_draft)
  seqlens           int32 [B]
  block_idx         int32 [B, Hkv, Tq, topk]
"""
import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinfllmv2.so")
BENCH_LIB_PATH = os.path.join(_HERE, "libinfllmv2_bench.so")   # + per-kernel timing and probes (include/infllmv2_bench.h)

OK = 0
OP_SELECT_PREFILL, OP_SELECT_DECODE, OP_ATTN_PREFILL, OP_ATTN_DECODE = 1, 2, 3, 4
OP_SELECT_VERIFY, OP_ATTN_VERIFY = 5, 6
OP_ATTN_BWD = 7
OP_DECODE_STEP = 8
OP_SELECT_SHARED = 9
OP_VERIFY_STEP = 10
MODE_PREFILL, MODE_DECODE = 0, 1

EXPORTS = ["infllmv2_status_string", "infllmv2_workspace_bytes", "infllmv2_compress_keys",
           "infllmv2_select_blocks", "infllmv2_sparse_attn_prefill", "infllmv2_sparse_attn_decode", "infllmv2_sparse_attn_decode_noalloc",
           "infllmv2_sparse_attn_bwd", "infllmv2_append_kv", "infllmv2_decode_step", "infllmv2_select_blocks_shared", "infllmv2_sparse_attn_prefill_shared", "infllmv2_verify_workspace_bytes", "infllmv2_append_kv_verify",
           "infllmv2_select_blocks_verify", "infllmv2_sparse_attn_verify", "infllmv2_verify_step",
           "infllmv2_block_scores"]
BENCH_EXPORTS = ["infllmv2_probe_peaks", "infllmv2_probe_detail", "infllmv2_timing_enable", "infllmv2_timing_read"]


class CParams(ctypes.Structure):
    _fields_ = [("head_dim", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("kernel_size", ctypes.c_int32), ("kernel_stride", ctypes.c_int32),
                ("topk", ctypes.c_int32), ("n_init_blocks", ctypes.c_int32),
                ("n_local_blocks", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("lse_coarse_ratio", ctypes.c_int32)]


class CTensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_b", ctypes.c_int64),
                ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64)]


@dataclass
class Params:
    """Hyper-parameters of section 2.1 (m = block_size, p = kernel_size, s = kernel_stride, k = topk)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    block_size: int = 64
    kernel_size: int = 32
    kernel_stride: int = 16
    topk: int = 16
    n_init_blocks: int = 1
    n_local_blocks: int = 2
    softmax_scale: float = None
    lse_coarse_ratio: int = 1      # rho of the approximate log-sum-exp (prefill selection); 1 = exact

    def __post_init__(self):
        if self.softmax_scale is None:
            self.softmax_scale = float(self.head_dim) ** -0.5

    def c(self):
        return CParams(self.head_dim, self.n_q_heads, self.n_kv_heads, self.block_size,
                       self.kernel_size, self.kernel_stride, self.topk, self.n_init_blocks,
                       self.n_local_blocks, self.softmax_scale, self.lse_coarse_ratio)


class InfLLMv2Error(RuntimeError):
    pass


_lib = None


def load_library(path=None):
    """Load libinfllmv2.so (built by paper_2506_07900_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("INFLLMV2_LIB") or LIB_PATH     # INFLLMV2_LIB: use another build of the library
    if not os.path.exists(path):
        raise InfLLMv2Error("HIP library not built: %s is missing (run python -m paper_2506_07900_amd.build)" % path)
    lib = ctypes.CDLL(path)
    i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    P, T = ctypes.POINTER(CParams), ctypes.POINTER(CTensor)
    lib.infllmv2_status_string.restype = ctypes.c_char_p
    lib.infllmv2_status_string.argtypes = [i32]
    lib.infllmv2_workspace_bytes.restype = sz
    lib.infllmv2_workspace_bytes.argtypes = [i32, P, i32, i32]
    lib.infllmv2_compress_keys.restype = i32
    lib.infllmv2_compress_keys.argtypes = [P, T, vp, i32, i32, i32, T, vp]
    lib.infllmv2_select_blocks.restype = i32
    lib.infllmv2_select_blocks.argtypes = [P, i32, T, T, vp, i32, i32, vp, vp, sz, vp]
    lib.infllmv2_block_scores.restype = i32
    lib.infllmv2_block_scores.argtypes = [P, T, T, vp, i32, i32, vp, i32, vp, sz, vp]
    lib.infllmv2_sparse_attn_prefill.restype = i32
    lib.infllmv2_sparse_attn_prefill.argtypes = [P, T, T, T, vp, i32, i32, vp, T, vp, vp, sz, vp]
    lib.infllmv2_sparse_attn_decode.restype = i32
    lib.infllmv2_sparse_attn_decode.argtypes = [P, T, T, T, vp, i32, i32, vp, T, vp, vp, sz, vp]
    lib.infllmv2_sparse_attn_decode_noalloc.restype = i32
    lib.infllmv2_sparse_attn_decode_noalloc.argtypes = [P, T, T, T, vp, i32, i32, vp, T, vp, vp]
    lib.infllmv2_sparse_attn_bwd.restype = i32
    lib.infllmv2_sparse_attn_bwd.argtypes = [P, T, T, T, T, T, vp, vp, i32, i32, vp, T, T, T, vp, sz, vp]
    lib.infllmv2_decode_step.restype = i32
    lib.infllmv2_decode_step.argtypes = [P, T, T, T, T, T, T, vp, i32, i32, vp, T, vp, vp, sz, vp]
    lib.infllmv2_select_blocks_shared.restype = i32
    lib.infllmv2_select_blocks_shared.argtypes = [P, T, T, vp, i32, i32, vp, vp, sz, vp]
    lib.infllmv2_sparse_attn_prefill_shared.restype = i32
    lib.infllmv2_sparse_attn_prefill_shared.argtypes = [P, T, T, T, vp, i32, i32, vp, T, vp, vp, sz, vp]
    lib.infllmv2_append_kv.restype = i32
    lib.infllmv2_append_kv.argtypes = [P, T, T, T, T, T, vp, i32, i32, vp]
    lib.infllmv2_verify_workspace_bytes.restype = sz
    lib.infllmv2_verify_workspace_bytes.argtypes = [i32, P, i32, i32, i32]
    lib.infllmv2_append_kv_verify.restype = i32
    lib.infllmv2_append_kv_verify.argtypes = [P, T, T, T, T, T, vp, i32, i32, i32, vp]
    lib.infllmv2_select_blocks_verify.restype = i32
    lib.infllmv2_select_blocks_verify.argtypes = [P, T, T, vp, i32, i32, i32, vp, vp, sz, vp]
    lib.infllmv2_verify_step.restype = i32
    lib.infllmv2_verify_step.argtypes = [P, T, T, T, T, T, T, vp, i32, i32, i32, vp, vp, T, vp, vp, sz, vp]
    lib.infllmv2_sparse_attn_verify.restype = i32
    lib.infllmv2_sparse_attn_verify.argtypes = [P, T, T, T, vp, i32, i32, i32, vp, vp, T, vp, vp, sz, vp]
    if hasattr(lib, "infllmv2_timing_enable"):            # the bench build
        lib.infllmv2_probe_peaks.restype = i32
        lib.infllmv2_probe_peaks.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp]
        lib.infllmv2_probe_detail.restype = i32
        lib.infllmv2_probe_detail.argtypes = [vp, sz, ctypes.POINTER(ctypes.c_double), vp]
        lib.infllmv2_timing_enable.restype = i32
        lib.infllmv2_timing_enable.argtypes = [i32]
        lib.infllmv2_timing_read.restype = i32
        lib.infllmv2_timing_read.argtypes = [i32, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float)]
    _lib = lib
    return lib


def load_bench_library():
    """Make libinfllmv2_bench.so the library every call of this module goes through: the same entry points,
    plus timing_enable / timing_read / probe_peaks.  For benchmarks; call it before anything else."""
    return load_library(BENCH_LIB_PATH)


def _bench_lib():
    lib = load_library()
    if not hasattr(lib, "infllmv2_timing_enable"):
        raise InfLLMv2Error("per-kernel timing and the probes are in libinfllmv2_bench.so only: call load_bench_library() first")
    return lib


def status_string(status):
    return load_library().infllmv2_status_string(int(status)).decode()


def _check(status, what):
    if status != OK:
        raise InfLLMv2Error("%s failed: %s (%d)" % (what, status_string(status), status))


def _bf16(t, ndim, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == ndim):
        raise InfLLMv2Error("%s must be a %d-d bf16 device tensor" % (name, ndim))
    if t.stride(-1) != 1:
        raise InfLLMv2Error("%s: head_dim axis must be contiguous" % name)
    return t


def _cache_desc(t, name):       # [B, Hkv, T, d]
    _bf16(t, 4, name)
    return CTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _query_desc(t, name):       # [B, T, Hq, d]
    _bf16(t, 4, name)
    return CTensor(t.data_ptr(), t.stride(0), t.stride(2), t.stride(1))


def _i32(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise InfLLMv2Error("%s must be a contiguous int32 device tensor" % name)
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def timing_enable(enable):
    _check(_bench_lib().infllmv2_timing_enable(1 if enable else 0), "infllmv2_timing_enable")


def timing_read(max_entries=256):
    """-> list of (kernel name, milliseconds) for the launches recorded since the last read."""
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_float * max_entries)()
    n = _bench_lib().infllmv2_timing_read(max_entries, names, ms)
    if n < 0:
        _check(n, "infllmv2_timing_read")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def num_kernels(seqlen, prm):
    """n_c(l): complete semantic kernels of a sequence of l tokens."""
    return 0 if seqlen < prm.kernel_size else (seqlen - prm.kernel_size) // prm.kernel_stride + 1


def workspace_bytes(op, prm, batch, max_seqlen):
    return int(load_library().infllmv2_workspace_bytes(op, ctypes.byref(prm.c()), batch, max_seqlen))


def _workspace(op, prm, batch, max_seqlen, workspace, device):
    need = workspace_bytes(op, prm, batch, max_seqlen)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def compress_keys(prm, k, seqlens, max_seqlen, ck=None, n_new_tokens=0):
    """k [B, Hkv, T, d] -> ck [B, Hkv, n_c(max_seqlen) (or more), d] (allocated if not given)."""
    lib = load_library()
    B, Hkv = k.shape[0], k.shape[1]
    if ck is None:
        ck = torch.zeros((B, Hkv, max(num_kernels(max_seqlen, prm), 1), k.shape[3]),
                         dtype=torch.bfloat16, device=k.device)
    kd, cd = _cache_desc(k, "k"), _cache_desc(ck, "ck")
    _check(lib.infllmv2_compress_keys(ctypes.byref(prm.c()), ctypes.byref(kd), _i32(seqlens, "seqlens").data_ptr(),
                                      B, max_seqlen, n_new_tokens, ctypes.byref(cd), _stream()),
           "infllmv2_compress_keys")
    return ck


def append_kv(prm, k_new, v_new, k, v, seqlens, max_seqlen, ck=None):
    """k_new, v_new [B, Hkv, 1, d] are written at cache position seqlens[b]-1; with ck the
    compressed key that the new token completes (if any) is written in the same launch."""
    lib = load_library()
    d = [_cache_desc(k_new, "k_new"), _cache_desc(v_new, "v_new"), _cache_desc(k, "k"), _cache_desc(v, "v")]
    ckd = ctypes.byref(_cache_desc(ck, "ck")) if ck is not None else None
    _check(lib.infllmv2_append_kv(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                  ctypes.byref(d[2]), ctypes.byref(d[3]), ckd,
                                  _i32(seqlens, "seqlens").data_ptr(), k.shape[0], max_seqlen, _stream()),
           "infllmv2_append_kv")


def probe_peaks(buf):
    """Launch the two probe kernels over the zero-filled uint8 device buffer `buf`;
    -> (flops of the MFMA probe, bytes of the stream probe).  Durations come from timing_read()."""
    lib = _bench_lib()
    fl, by = ctypes.c_double(), ctypes.c_double()
    _check(lib.infllmv2_probe_peaks(buf.data_ptr(), buf.numel(), ctypes.byref(fl), ctypes.byref(by), _stream()),
           "infllmv2_probe_peaks")
    return fl.value, by.value


def block_scores(prm, q, ck, seqlens, max_seqlen, scores=None, workspace=None):
    """-> fp32 [B, Hkv, max_seqlen, n_blocks]: the block scores of the candidate blocks of every prefill
    query (entries of other blocks keep the NaN the buffer is created with)."""
    lib = load_library()
    B = q.shape[0]
    nb = (max_seqlen + prm.block_size - 1) // prm.block_size
    if scores is None:
        scores = torch.full((B, prm.n_kv_heads, max_seqlen, nb), float("nan"), dtype=torch.float32, device=q.device)
    ws, ws_bytes = _workspace(OP_SELECT_PREFILL, prm, B, max_seqlen, workspace, q.device)
    qd, ckd = _query_desc(q, "q"), _cache_desc(ck, "ck")
    _check(lib.infllmv2_block_scores(ctypes.byref(prm.c()), ctypes.byref(qd), ctypes.byref(ckd),
                                     _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen, scores.data_ptr(),
                                     scores.stride(2), ws.data_ptr(), ws_bytes, _stream()),
           "infllmv2_block_scores")
    return scores


def probe_detail(buf):
    """Launch the issue and fragment probes over the zero-filled uint8 device buffer `buf` -> the 7 work
    figures of infllmv2_probe_detail (groups per SIMD x 5, bytes x 2).  Durations come from timing_read()."""
    lib = _bench_lib()
    work = (ctypes.c_double * 7)()
    _check(lib.infllmv2_probe_detail(buf.data_ptr(), buf.numel(), work, _stream()), "infllmv2_probe_detail")
    return [float(w) for w in work]


def select_blocks(prm, mode, q, ck, seqlens, max_seqlen, block_idx=None, workspace=None):
    """-> block_idx int32 [B, Hkv, Tq, topk] (Tq = max_seqlen in prefill, 1 in decode)."""
    lib = load_library()
    B = q.shape[0]
    n_q = max_seqlen if mode == MODE_PREFILL else 1
    if block_idx is None:
        block_idx = torch.full((B, prm.n_kv_heads, n_q, prm.topk), -1, dtype=torch.int32, device=q.device)
    op = OP_SELECT_PREFILL if mode == MODE_PREFILL else OP_SELECT_DECODE
    workspace, ws_bytes = _workspace(op, prm, B, max_seqlen, workspace, q.device)
    qd, cd = _query_desc(q, "q"), _cache_desc(ck, "ck")
    _check(lib.infllmv2_select_blocks(ctypes.byref(prm.c()), mode, ctypes.byref(qd), ctypes.byref(cd),
                                      _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen,
                                      _i32(block_idx, "block_idx").data_ptr(), workspace.data_ptr(),
                                      ws_bytes, _stream()), "infllmv2_select_blocks")
    return block_idx


def sparse_attn_prefill(prm, q, k, v, seqlens, max_seqlen, block_idx, out=None, lse=None, workspace=None):
    """-> out bf16 [B, T, Hq, d], lse fp32 [B, T, Hq]."""
    lib = load_library()
    B = q.shape[0]
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, max_seqlen, prm.n_q_heads), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _workspace(OP_ATTN_PREFILL, prm, B, max_seqlen, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out")]
    _check(lib.infllmv2_sparse_attn_prefill(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                            ctypes.byref(d[2]), _i32(seqlens, "seqlens").data_ptr(), B,
                                            max_seqlen, _i32(block_idx, "block_idx").data_ptr(),
                                            ctypes.byref(d[3]), lse.data_ptr(), workspace.data_ptr(),
                                            ws_bytes, _stream()), "infllmv2_sparse_attn_prefill")
    return out, lse


def sparse_attn_decode(prm, q, k, v, seqlens, max_seqlen, block_idx, out=None, lse=None, workspace=None):
    """q [B, 1, Hq, d] -> out bf16 [B, 1, Hq, d], lse fp32 [B, Hq]."""
    lib = load_library()
    B = q.shape[0]
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, prm.n_q_heads), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _workspace(OP_ATTN_DECODE, prm, B, max_seqlen, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out")]
    _check(lib.infllmv2_sparse_attn_decode(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                           ctypes.byref(d[2]), _i32(seqlens, "seqlens").data_ptr(), B,
                                           max_seqlen, _i32(block_idx, "block_idx").data_ptr(),
                                           ctypes.byref(d[3]), lse.data_ptr(), workspace.data_ptr(),
                                           ws_bytes, _stream()), "infllmv2_sparse_attn_decode")
    return out, lse


def sparse_attn_decode_noalloc(prm, q, k, v, seqlens, max_seqlen, block_idx, out, lse):
    """sparse_attn_decode on the library's fixed scratch array: no workspace, and this wrapper creates no
    tensor either (out [B, 1, Hq, d] bf16 and lse [B, Hq] fp32 are the caller's)."""
    lib = load_library()
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out")]
    _check(lib.infllmv2_sparse_attn_decode_noalloc(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                                   ctypes.byref(d[2]), _i32(seqlens, "seqlens").data_ptr(),
                                                   q.shape[0], max_seqlen, _i32(block_idx, "block_idx").data_ptr(),
                                                   ctypes.byref(d[3]), lse.data_ptr(), _stream()),
           "infllmv2_sparse_attn_decode_noalloc")
    return out, lse


# ---- draft verification (section 4.1, "InfLLM v2 for Target Model") ---------------------------------

def verify_workspace_bytes(op, prm, batch, max_seqlen, n_draft):
    return int(load_library().infllmv2_verify_workspace_bytes(op, ctypes.byref(prm.c()), batch, max_seqlen, n_draft))


def _verify_workspace(op, prm, batch, max_seqlen, n_draft, workspace, device):
    need = verify_workspace_bytes(op, prm, batch, max_seqlen, n_draft)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def append_kv_verify(prm, k_new, v_new, k, v, seqlens, max_seqlen, ck=None):
    """k_new, v_new [B, Hkv, n_draft, d] are written at cache rows seqlens[b]-n_draft .. seqlens[b]-1;
    with ck the compressed keys those rows complete are written too."""
    lib = load_library()
    d = [_cache_desc(k_new, "k_new"), _cache_desc(v_new, "v_new"), _cache_desc(k, "k"), _cache_desc(v, "v")]
    ckd = ctypes.byref(_cache_desc(ck, "ck")) if ck is not None else None
    _check(lib.infllmv2_append_kv_verify(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                         ctypes.byref(d[2]), ctypes.byref(d[3]), ckd,
                                         _i32(seqlens, "seqlens").data_ptr(), k.shape[0], max_seqlen,
                                         k_new.shape[2], _stream()), "infllmv2_append_kv_verify")


def select_blocks_verify(prm, q, ck, seqlens, max_seqlen, block_idx=None, workspace=None):
    """q [B, n_draft, Hq, d] -> block_idx int32 [B, Hkv, n_draft, topk]."""
    lib = load_library()
    B, n = q.shape[0], q.shape[1]
    if block_idx is None:
        block_idx = torch.full((B, prm.n_kv_heads, n, prm.topk), -1, dtype=torch.int32, device=q.device)
    workspace, ws_bytes = _verify_workspace(OP_SELECT_VERIFY, prm, B, max_seqlen, n, workspace, q.device)
    qd, cd = _query_desc(q, "q"), _cache_desc(ck, "ck")
    _check(lib.infllmv2_select_blocks_verify(ctypes.byref(prm.c()), ctypes.byref(qd), ctypes.byref(cd),
                                             _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen, n,
                                             _i32(block_idx, "block_idx").data_ptr(), workspace.data_ptr(),
                                             ws_bytes, _stream()), "infllmv2_select_blocks_verify")
    return block_idx


def sparse_attn_verify(prm, q, k, v, seqlens, max_seqlen, block_idx, tree_mask=None, out=None, lse=None,
                       workspace=None):
    """q [B, n_draft, Hq, d]; tree_mask int64 device tensor [B, n_draft] holding the uint64 mask words
    (None = causal chain) -> out bf16 [B, n_draft, Hq, d], lse fp32 [B, n_draft, Hq]."""
    lib = load_library()
    B, n = q.shape[0], q.shape[1]
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, n, prm.n_q_heads), dtype=torch.float32, device=q.device)
    mask_ptr = None
    if tree_mask is not None:
        if not (tree_mask.is_cuda and tree_mask.dtype == torch.int64 and tree_mask.is_contiguous()
                and tuple(tree_mask.shape) == (B, n)):
            raise InfLLMv2Error("tree_mask must be a contiguous int64 device tensor [B, n_draft]")
        mask_ptr = tree_mask.data_ptr()
    workspace, ws_bytes = _verify_workspace(OP_ATTN_VERIFY, prm, B, max_seqlen, n, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out")]
    _check(lib.infllmv2_sparse_attn_verify(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                           ctypes.byref(d[2]), _i32(seqlens, "seqlens").data_ptr(), B,
                                           max_seqlen, n, mask_ptr, _i32(block_idx, "block_idx").data_ptr(),
                                           ctypes.byref(d[3]), lse.data_ptr(), workspace.data_ptr(),
                                           ws_bytes, _stream()), "infllmv2_sparse_attn_verify")
    return out, lse


def verify_step(prm, q, k_new, v_new, k, v, ck, seqlens, max_seqlen, tree_mask=None, block_idx=None, out=None,
                lse=None, workspace=None):
    """One verification step in one call: append_kv_verify (with ck) + select_blocks_verify + sparse_attn_verify.
    q [B, n_draft, Hq, d]; k_new, v_new [B, Hkv, n_draft, d] -> block_idx [B, Hkv, n_draft, topk], out, lse."""
    lib = load_library()
    B, n = q.shape[0], q.shape[1]
    if block_idx is None:
        block_idx = torch.full((B, prm.n_kv_heads, n, prm.topk), -1, dtype=torch.int32, device=q.device)
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, n, prm.n_q_heads), dtype=torch.float32, device=q.device)
    mask_ptr = None
    if tree_mask is not None:
        if not (tree_mask.is_cuda and tree_mask.dtype == torch.int64 and tree_mask.is_contiguous()
                and tuple(tree_mask.shape) == (B, n)):
            raise InfLLMv2Error("tree_mask must be a contiguous int64 device tensor [B, n_draft]")
        mask_ptr = tree_mask.data_ptr()
    workspace, ws_bytes = _verify_workspace(OP_VERIFY_STEP, prm, B, max_seqlen, n, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k_new, "k_new"), _cache_desc(v_new, "v_new"), _cache_desc(k, "k"),
         _cache_desc(v, "v"), _cache_desc(ck, "ck"), _query_desc(out, "out")]
    _check(lib.infllmv2_verify_step(ctypes.byref(prm.c()), *[ctypes.byref(x) for x in d[:6]],
                                    _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen, n, mask_ptr,
                                    _i32(block_idx, "block_idx").data_ptr(), ctypes.byref(d[6]), lse.data_ptr(),
                                    workspace.data_ptr(), ws_bytes, _stream()), "infllmv2_verify_step")
    return block_idx, out, lse


def sparse_attn_bwd(prm, q, k, v, out, dout, lse, seqlens, max_seqlen, block_idx, dq=None, dk=None, dv=None,
                    workspace=None):
    """Backward of sparse_attn_prefill with the block sets fixed -> dq [B, T, Hq, d], dk, dv [B, Hkv, T, d] (bf16)."""
    lib = load_library()
    B = q.shape[0]
    dq = torch.zeros_like(q) if dq is None else dq
    dk = torch.zeros_like(k) if dk is None else dk
    dv = torch.zeros_like(v) if dv is None else dv
    workspace, ws_bytes = _workspace(OP_ATTN_BWD, prm, B, max_seqlen, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out"),
         _query_desc(dout, "dout"), _query_desc(dq, "dq"), _cache_desc(dk, "dk"), _cache_desc(dv, "dv")]
    if not (lse.is_cuda and lse.dtype == torch.float32 and lse.is_contiguous()):
        raise InfLLMv2Error("lse must be a contiguous fp32 device tensor")
    _check(lib.infllmv2_sparse_attn_bwd(ctypes.byref(prm.c()), *[ctypes.byref(x) for x in d[:5]], lse.data_ptr(),
                                        _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen,
                                        _i32(block_idx, "block_idx").data_ptr(), *[ctypes.byref(x) for x in d[5:]],
                                        workspace.data_ptr(), ws_bytes, _stream()), "infllmv2_sparse_attn_bwd")
    return dq, dk, dv


def decode_step(prm, q, k_new, v_new, k, v, ck, seqlens, max_seqlen, block_idx=None, out=None, lse=None,
                workspace=None):
    """append_kv (with ck) + select_blocks(MODE_DECODE) + sparse_attn_decode in one call, five launches.
    -> block_idx [B, Hkv, 1, topk], out [B, 1, Hq, d], lse [B, Hq]."""
    lib = load_library()
    B = q.shape[0]
    if block_idx is None:
        block_idx = torch.full((B, prm.n_kv_heads, 1, prm.topk), -1, dtype=torch.int32, device=q.device)
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, prm.n_q_heads), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _workspace(OP_DECODE_STEP, prm, B, max_seqlen, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k_new, "k_new"), _cache_desc(v_new, "v_new"), _cache_desc(k, "k"),
         _cache_desc(v, "v"), _cache_desc(ck, "ck"), _query_desc(out, "out")]
    _check(lib.infllmv2_decode_step(ctypes.byref(prm.c()), *[ctypes.byref(x) for x in d[:6]],
                                    _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen,
                                    _i32(block_idx, "block_idx").data_ptr(), ctypes.byref(d[6]), lse.data_ptr(),
                                    workspace.data_ptr(), ws_bytes, _stream()), "infllmv2_decode_step")
    return block_idx, out, lse


def select_blocks_shared(prm, q, ck, seqlens, max_seqlen, block_idx=None, workspace=None):
    """Query-block-shared selection (comparison variant, not the report's method)
    -> block_idx int32 [B, Hkv, ceil(max_seqlen / 64), topk]."""
    lib = load_library()
    B = q.shape[0]
    n_qb = (max_seqlen + prm.block_size - 1) // prm.block_size
    if block_idx is None:
        block_idx = torch.full((B, prm.n_kv_heads, n_qb, prm.topk), -1, dtype=torch.int32, device=q.device)
    workspace, ws_bytes = _workspace(OP_SELECT_SHARED, prm, B, max_seqlen, workspace, q.device)
    qd, cd = _query_desc(q, "q"), _cache_desc(ck, "ck")
    _check(lib.infllmv2_select_blocks_shared(ctypes.byref(prm.c()), ctypes.byref(qd), ctypes.byref(cd),
                                             _i32(seqlens, "seqlens").data_ptr(), B, max_seqlen,
                                             _i32(block_idx, "block_idx").data_ptr(), workspace.data_ptr(),
                                             ws_bytes, _stream()), "infllmv2_select_blocks_shared")
    return block_idx


def sparse_attn_prefill_shared(prm, q, k, v, seqlens, max_seqlen, block_idx, out=None, lse=None, workspace=None):
    """Attention for block sets shared per 64-token query block (comparison variant); block_idx
    [B, Hkv, ceil(T/64), topk] -> out bf16 [B, T, Hq, d], lse fp32 [B, T, Hq]."""
    lib = load_library()
    B = q.shape[0]
    if out is None:
        out = torch.zeros_like(q)
    if lse is None:
        lse = torch.zeros((B, max_seqlen, prm.n_q_heads), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _workspace(OP_ATTN_PREFILL, prm, B, max_seqlen, workspace, q.device)
    d = [_query_desc(q, "q"), _cache_desc(k, "k"), _cache_desc(v, "v"), _query_desc(out, "out")]
    _check(lib.infllmv2_sparse_attn_prefill_shared(ctypes.byref(prm.c()), ctypes.byref(d[0]), ctypes.byref(d[1]),
                                                   ctypes.byref(d[2]), _i32(seqlens, "seqlens").data_ptr(), B,
                                                   max_seqlen, _i32(block_idx, "block_idx").data_ptr(),
                                                   ctypes.byref(d[3]), lse.data_ptr(), workspace.data_ptr(),
                                                   ws_bytes, _stream()), "infllmv2_sparse_attn_prefill_shared")
    return out, lse
