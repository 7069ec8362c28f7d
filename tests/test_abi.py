"""CPU checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments with a status code before any HIP call (so this runs without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2506_07900_amd import binding
from paper_2506_07900_amd.binding import CParams, CTensor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INVALID, UNSUPPORTED, WORKSPACE = -1, -2, -3


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_07900_amd import build
        build.build()
    return binding.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "infllmv2.h")).read()
    declared = sorted(set(re.findall(r"\b(infllmv2_[a-z_]+)\s*\(", text)))
    assert set(declared) == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_measurement_entry_points_live_in_the_bench_library_only(lib):
    # per-kernel timing (process-wide state, synchronises) and the probe kernels are not product code:
    # they are declared in their own header and exported by libinfllmv2_bench.so, which also has
    # every entry point of the library proper
    text = open(os.path.join(ROOT, "include", "infllmv2_bench.h")).read()
    declared = sorted(set(re.findall(r"\b(infllmv2_[a-z_]+)\s*\(", text)))
    assert set(declared) == set(binding.BENCH_EXPORTS)
    for name in declared:
        assert not hasattr(lib, name), name
    assert os.path.exists(binding.BENCH_LIB_PATH)
    bench = ctypes.CDLL(binding.BENCH_LIB_PATH)
    for name in binding.EXPORTS + binding.BENCH_EXPORTS:
        assert hasattr(bench, name), name
    with pytest.raises(binding.InfLLMv2Error):
        binding.timing_enable(True)


def test_header_is_plain_c():
    # the boundary is a C ABI: the headers have to compile as strict C99 (and as C++) on their own
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no host C compiler")
    for name in ("infllmv2.h", "infllmv2_bench.h"):
        hdr = os.path.join(ROOT, "include", name)
        for lang, std in (("c", "-std=c99"), ("c++", "-std=c++17")):
            r = subprocess.run(["gcc", "-x", lang, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", hdr],
                               capture_output=True, text=True)
            assert r.returncode == 0, r.stderr


def test_struct_layout_matches_header():
    assert ctypes.sizeof(CParams) == 44 and ctypes.sizeof(CTensor) == 32      # 10 int32 + 1 float; 1 pointer + 3 int64


def good_params(**kw):
    p = dict(head_dim=128, n_q_heads=32, n_kv_heads=2, block_size=64, kernel_size=32, kernel_stride=16,
             topk=16, n_init_blocks=1, n_local_blocks=2, softmax_scale=128 ** -0.5)
    p.update(kw)
    return CParams(**p)


FAKE = 0x10000   # non-null, 256-byte aligned; never dereferenced because validation fails first


def tensor(ptr=FAKE, sb=1 << 20, sh=1 << 16, st=128):
    return CTensor(ptr, sb, sh, st)


def call_compress(lib, prm, k=None, ck=None, seqlens=FAKE, batch=1, max_seqlen=1024):
    k = k or tensor()
    ck = ck or tensor()
    return lib.infllmv2_compress_keys(ctypes.byref(prm) if prm else None, ctypes.byref(k), seqlens, batch,
                                      max_seqlen, 0, ctypes.byref(ck), None)


def test_status_strings(lib):
    assert lib.infllmv2_status_string(0) == b"ok"
    for s in (-1, -2, -3, -4):
        assert lib.infllmv2_status_string(s) not in (b"ok", b"unknown status")
    assert lib.infllmv2_status_string(-99) == b"unknown status"


def test_parameter_validation(lib):
    assert call_compress(lib, None) == INVALID
    assert call_compress(lib, good_params(n_q_heads=30, n_kv_heads=4)) == INVALID      # ragged head ratio
    assert call_compress(lib, good_params(topk=2)) == INVALID                           # fewer than forced
    assert call_compress(lib, good_params(softmax_scale=0.0)) == INVALID
    assert call_compress(lib, good_params(head_dim=64)) == UNSUPPORTED
    assert call_compress(lib, good_params(block_size=128)) == UNSUPPORTED
    assert call_compress(lib, good_params(kernel_size=16)) == UNSUPPORTED
    assert call_compress(lib, good_params(n_q_heads=64, n_kv_heads=2)) == UNSUPPORTED  # G = 32
    assert call_compress(lib, good_params(topk=65)) == UNSUPPORTED
    # approximate log-sum-exp: ratios 2 and 4, G = 16, and a visible coarse kernel for every query
    # that has candidate blocks
    assert call_compress(lib, good_params(lse_coarse_ratio=-1)) == INVALID
    assert call_compress(lib, good_params(lse_coarse_ratio=3)) == UNSUPPORTED
    assert call_compress(lib, good_params(lse_coarse_ratio=8)) == UNSUPPORTED
    assert call_compress(lib, good_params(lse_coarse_ratio=2, n_q_heads=16, n_kv_heads=2)) == UNSUPPORTED   # G = 8
    assert call_compress(lib, good_params(lse_coarse_ratio=4, n_init_blocks=0, n_local_blocks=1, topk=4)) == UNSUPPORTED
    assert call_compress(lib, good_params(), seqlens=None) == INVALID
    assert call_compress(lib, good_params(), k=tensor(ptr=None)) == INVALID
    assert call_compress(lib, good_params(), k=tensor(ptr=FAKE + 2)) == INVALID        # misaligned
    assert call_compress(lib, good_params(), ck=tensor(st=100)) == INVALID             # stride not /8
    assert call_compress(lib, good_params(), batch=-1) == INVALID
    assert call_compress(lib, good_params(), max_seqlen=-5) == INVALID


def test_workspace_validation(lib):
    prm = good_params()
    need = lib.infllmv2_workspace_bytes(binding.OP_SELECT_PREFILL, ctypes.byref(prm), 1, 4096)
    # fp32 log-sum-exp per (token, head) + fragment-major copy of the compressed keys (4 KiB per
    # 16 kernels: 254 kernels = 16 tiles, plus the tile a last candidate block may reach into); no
    # score matrix: linear in max_seqlen
    assert need == 4096 * 32 * 4 + 2 * 17 * 4096
    need_long = lib.infllmv2_workspace_bytes(binding.OP_SELECT_PREFILL, ctypes.byref(prm), 1, 32 * 4096)
    assert need_long <= 33 * need
    # the query-block-shared comparison variant still stores fp32 block scores per (token, kv head, block)
    # and per (query block, kv head, block)
    need_shared = lib.infllmv2_workspace_bytes(binding.OP_SELECT_SHARED, ctypes.byref(prm), 1, 4096)
    assert need_shared == need + 2 * 4096 * 64 * 4 + 2 * 64 * 64 * 4
    assert lib.infllmv2_workspace_bytes(binding.OP_ATTN_PREFILL, ctypes.byref(prm), 1, 4096) == 2 * 64 * 32768
    assert lib.infllmv2_workspace_bytes(binding.OP_ATTN_DECODE, ctypes.byref(prm), 2, 4096) > 0
    assert lib.infllmv2_workspace_bytes(99, ctypes.byref(prm), 1, 4096) == 0
    q, ck = tensor(), tensor()
    args = (ctypes.byref(prm), 0, ctypes.byref(q), ctypes.byref(ck), FAKE, 1, 4096, FAKE)
    assert lib.infllmv2_select_blocks(*args, None, 0, None) == WORKSPACE
    assert lib.infllmv2_select_blocks(*args, FAKE, need - 1, None) == WORKSPACE
    assert lib.infllmv2_select_blocks(*args, FAKE + 16, need, None) == WORKSPACE        # not 256-aligned
    bad_mode = (ctypes.byref(prm), 7, ctypes.byref(q), ctypes.byref(ck), FAKE, 1, 4096, FAKE)
    assert lib.infllmv2_select_blocks(*bad_mode, FAKE, need, None) == INVALID
    dec = (ctypes.byref(prm), 1, ctypes.byref(q), ctypes.byref(ck), FAKE, 1, 1 << 20, FAKE)
    assert lib.infllmv2_select_blocks(*dec, FAKE, 1 << 40, None) == UNSUPPORTED         # decode context cap
    o = tensor()
    assert lib.infllmv2_sparse_attn_decode(ctypes.byref(prm), ctypes.byref(q), ctypes.byref(q), ctypes.byref(q),
                                           FAKE, 1, 4096, FAKE, ctypes.byref(o), FAKE, None, 0, None) == WORKSPACE
    assert lib.infllmv2_sparse_attn_prefill(ctypes.byref(prm), ctypes.byref(q), ctypes.byref(q), ctypes.byref(q),
                                            FAKE, 1, 4096, None, ctypes.byref(o), FAKE, None, 0, None) == INVALID
    assert lib.infllmv2_sparse_attn_prefill(ctypes.byref(prm), ctypes.byref(q), ctypes.byref(q), ctypes.byref(q),
                                            FAKE, 1, 4096, FAKE, ctypes.byref(o), FAKE, None, 0, None) == WORKSPACE


def test_noalloc_decode_validation(lib):
    # the fixed-scratch variant validates like the workspace one and refuses sizes beyond its array, all
    # on the host before any HIP call
    prm, q, o = good_params(), tensor(), tensor()
    P, Q, O = ctypes.byref(prm), ctypes.byref(q), ctypes.byref(o)
    f = lib.infllmv2_sparse_attn_decode_noalloc
    assert f(P, Q, Q, Q, None, 1, 4096, FAKE, O, FAKE, None) == INVALID                  # no seqlens
    assert f(P, Q, Q, Q, FAKE, 1, 4096, FAKE, O, None, None) == INVALID                  # no lse
    assert f(P, Q, Q, Q, FAKE, -1, 4096, FAKE, O, FAKE, None) == INVALID
    assert f(P, Q, Q, Q, FAKE, 17, 4096, FAKE, O, FAKE, None) == UNSUPPORTED             # 17*32*16*520 B > 4 MiB
    bad = good_params(head_dim=64)
    assert f(ctypes.byref(bad), Q, Q, Q, FAKE, 1, 4096, FAKE, O, FAKE, None) == UNSUPPORTED


def test_append_kv_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    bad = tensor(st=100)                                                                 # stride not /8
    assert lib.infllmv2_append_kv(P, T, T, T, T, None, None, 1, 4096, None) == INVALID   # no seqlens
    assert lib.infllmv2_append_kv(P, T, T, T, T, ctypes.byref(bad), FAKE, 1, 4096, None) == INVALID
    assert lib.infllmv2_append_kv(P, None, T, T, T, None, FAKE, 1, 4096, None) == INVALID
    assert lib.infllmv2_append_kv(P, T, T, T, T, None, FAKE, 0, 4096, None) == 0         # empty batch: nothing to do


def test_verify_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    ws = lib.infllmv2_verify_workspace_bytes
    # 16 query rows: two (max, sum) partial sets of 2 chunks x 32 heads + fp32 scores of 64 blocks x 2 kv heads
    assert ws(binding.OP_SELECT_VERIFY, P, 2, 4096, 8) == 2 * 16 * 32 * 2 * 8 + 16 * 2 * 64 * 4
    assert ws(binding.OP_ATTN_VERIFY, P, 1, 4096, 1) == lib.infllmv2_workspace_bytes(binding.OP_ATTN_DECODE, P, 1, 4096)
    assert ws(binding.OP_ATTN_VERIFY, P, 1, 4096, 0) == 0 and ws(binding.OP_ATTN_VERIFY, P, 1, 4096, 65) == 0
    assert ws(binding.OP_SELECT_DECODE, P, 1, 4096, 4) == 0                              # not a verify stage
    sel = lambda n, w=FAKE, wb=1 << 40: lib.infllmv2_select_blocks_verify(P, T, T, FAKE, 1, 4096, n, FAKE, w, wb, None)
    assert sel(0) == INVALID and sel(-3) == INVALID
    assert sel(65) == UNSUPPORTED                                                        # one uint64 word per token
    assert sel(8, None, 0) == WORKSPACE
    assert lib.infllmv2_select_blocks_verify(P, T, T, FAKE, 16384, 4096, 4, FAKE, FAKE, 1 << 40, None) == UNSUPPORTED
    att = lambda n, mask=None, w=FAKE, wb=1 << 40: lib.infllmv2_sparse_attn_verify(
        P, T, T, T, FAKE, 1, 4096, n, mask, FAKE, T, FAKE, w, wb, None)
    assert att(0) == INVALID and att(65) == UNSUPPORTED
    assert att(4, FAKE + 4) == INVALID                                                   # mask words 8-byte aligned
    assert att(4, None, None, 0) == WORKSPACE
    app = lambda n, sl=FAKE: lib.infllmv2_append_kv_verify(P, T, T, T, T, None, sl, 1, 4096, n, None)
    assert app(0) == INVALID and app(65) == UNSUPPORTED and app(4, None) == INVALID
    assert lib.infllmv2_append_kv_verify(P, T, T, T, T, None, FAKE, 0, 4096, 4, None) == 0


def test_backward_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    need = lib.infllmv2_workspace_bytes(binding.OP_ATTN_BWD, P, 1, 4096)
    assert need > 2 * 64 * 3 * 16384                                                    # at least the packed blocks
    call = lambda lse=FAKE, idx=FAKE, w=FAKE, wb=1 << 40, dq=T: lib.infllmv2_sparse_attn_bwd(
        P, T, T, T, T, T, lse, FAKE, 1, 4096, idx, dq, T, T, w, wb, None)
    assert call(lse=None) == INVALID and call(idx=None) == INVALID and call(dq=None) == INVALID
    assert call(w=None, wb=0) == WORKSPACE and call(wb=need - 1) == WORKSPACE and call(w=FAKE + 16) == WORKSPACE
    assert lib.infllmv2_sparse_attn_bwd(P, T, T, T, T, T, FAKE, FAKE, 0, 4096, FAKE, T, T, T, FAKE, 1 << 40, None) == 0
    far = tensor()                                                                      # heads of a group too far apart
    far.stride_h = 1 << 28
    assert lib.infllmv2_sparse_attn_bwd(P, ctypes.byref(far), T, T, T, T, FAKE, FAKE, 1, 4096, FAKE, T, T, T, FAKE, 1 << 40,
                                        None) == UNSUPPORTED


def test_decode_step_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    need = lib.infllmv2_workspace_bytes(binding.OP_DECODE_STEP, P, 2, 4096)
    assert need == (lib.infllmv2_workspace_bytes(binding.OP_SELECT_DECODE, P, 2, 4096) +
                    lib.infllmv2_workspace_bytes(binding.OP_ATTN_DECODE, P, 2, 4096))
    call = lambda q=T, sl=FAKE, w=FAKE, wb=1 << 40, ms=4096: lib.infllmv2_decode_step(
        P, q, T, T, T, T, T, sl, 2, ms, FAKE, T, FAKE, w, wb, None)
    assert call(q=None) == INVALID and call(sl=None) == INVALID
    assert call(w=None, wb=0) == WORKSPACE and call(wb=need - 1) == WORKSPACE
    assert call(ms=1 << 20) == UNSUPPORTED                                               # decode context cap
    assert lib.infllmv2_decode_step(P, T, T, T, T, T, T, FAKE, 0, 4096, FAKE, T, FAKE, FAKE, 1 << 40, None) == 0


def test_verify_step_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    ws = lib.infllmv2_verify_workspace_bytes
    need = ws(binding.OP_VERIFY_STEP, P, 2, 4096, 8)
    assert need == ws(binding.OP_SELECT_VERIFY, P, 2, 4096, 8) + ws(binding.OP_ATTN_VERIFY, P, 2, 4096, 8) > 0
    assert ws(binding.OP_VERIFY_STEP, P, 2, 4096, 65) == 0 and ws(binding.OP_VERIFY_STEP, P, 2, 1 << 20, 8) == 0
    call = lambda n=8, q=T, ck=T, sl=FAKE, mask=None, w=FAKE, wb=1 << 40, ms=4096: lib.infllmv2_verify_step(
        P, q, T, T, T, T, ck, sl, 2, ms, n, mask, FAKE, T, FAKE, w, wb, None)
    assert call(n=0) == INVALID and call(n=65) == UNSUPPORTED
    assert call(q=None) == INVALID and call(ck=None) == INVALID and call(sl=None) == INVALID
    assert call(mask=FAKE + 4) == INVALID                                                # mask words 8-byte aligned
    assert call(w=None, wb=0) == WORKSPACE and call(wb=need - 1) == WORKSPACE and call(w=FAKE + 16) == WORKSPACE
    assert call(ms=1 << 20) == UNSUPPORTED                                               # decode context cap
    assert lib.infllmv2_verify_step(P, T, T, T, T, T, T, FAKE, 0, 4096, 8, None, FAKE, T, FAKE, FAKE, 1 << 40,
                                    None) == 0                                           # empty batch: nothing to do


def test_shared_variant_validation(lib):
    prm, t = good_params(), tensor()
    P, T = ctypes.byref(prm), ctypes.byref(t)
    need = lib.infllmv2_workspace_bytes(binding.OP_SELECT_SHARED, P, 1, 4096)
    # the per-token selection's scratch plus fp32 scores of 4096 tokens x 64 blocks x 2 kv heads (this
    # variant averages stored scores) and of 64 query blocks x 64 blocks x 2 kv heads
    assert need == (lib.infllmv2_workspace_bytes(binding.OP_SELECT_PREFILL, P, 1, 4096) + 2 * 4096 * 64 * 4 +
                    2 * 64 * 64 * 4)
    sel = lambda w=FAKE, wb=1 << 40, idx=FAKE: lib.infllmv2_select_blocks_shared(P, T, T, FAKE, 1, 4096, idx, w, wb, None)
    assert sel(idx=None) == INVALID and sel(w=None, wb=0) == WORKSPACE and sel(wb=need - 1) == WORKSPACE
    att = lambda w=FAKE, wb=1 << 40, idx=FAKE: lib.infllmv2_sparse_attn_prefill_shared(
        P, T, T, T, FAKE, 1, 4096, idx, T, FAKE, w, wb, None)
    assert att(idx=None) == INVALID and att(w=None, wb=0) == WORKSPACE


def test_binding_fails_loudly_without_library(tmp_path):
    with pytest.raises(binding.InfLLMv2Error):
        binding.load_library(str(tmp_path / "missing.so"))
