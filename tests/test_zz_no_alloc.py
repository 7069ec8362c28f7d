"""GPU test of infllmv2_sparse_attn_decode_noalloc, the decode attention on the library's fixed scratch
array (for callers that cannot allocate): two calls in a row through the C ABI, the second with a
smaller input, each bit-equal to infllmv2_sparse_attn_decode on the same arguments.  Collected last
(the file name sorts after the others)."""
import numpy as np
import pytest
import torch

from paper_2506_07900_amd import binding, synth
from util import to_dev

pytestmark = pytest.mark.gpu


def _case(seed, seqlens, Hq, Hkv, topk):
    B, T = len(seqlens), max(seqlens)
    d = 128
    q = np.zeros((B, 1, Hq, d), np.uint16)
    k = np.zeros((B, Hkv, T, d), np.uint16)
    v = np.zeros((B, Hkv, T, d), np.uint16)
    for b, l in enumerate(seqlens):
        x = synth.make_sequence(seed + b, l, Hq, Hkv, n_planted=2)
        q[b, 0], k[b, :, :l], v[b, :, :l] = x.q[l - 1], x.k, x.v
    prm = binding.Params(Hq, Hkv, topk=topk)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    sl = torch.tensor(seqlens, dtype=torch.int32, device="cuda")
    ck = binding.compress_keys(prm, kd, sl, T)
    idx = binding.select_blocks(prm, binding.MODE_DECODE, qd, ck, sl, T)
    return prm, qd, kd, vd, sl, T, idx


def test_noalloc_decode_matches_the_workspace_entry_point_twice():
    for seed, seqlens, Hq, Hkv, topk in [(5, [3000, 1077, 64, 33, 1, 700], 32, 2, 16), (9, [500, 129], 8, 2, 6)]:
        print("case noalloc", seqlens, Hq, Hkv, topk, flush=True)
        prm, qd, kd, vd, sl, T, idx = _case(seed, seqlens, Hq, Hkv, topk)
        want_o, want_l = binding.sparse_attn_decode(prm, qd, kd, vd, sl, T, idx)
        out = torch.full_like(qd, 7.0)
        lse = torch.full((len(seqlens), Hq), 7.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        binding.sparse_attn_decode_noalloc(prm, qd, kd, vd, sl, T, idx, out, lse)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out.view(torch.int16), want_o.view(torch.int16))
        assert torch.equal(lse.view(torch.int32), want_l.view(torch.int32))


def test_noalloc_decode_rejects_sizes_beyond_the_array():
    prm, qd, kd, vd, sl, T, idx = _case(3, [200], 32, 2, 16)
    B = 64                                                   # 64 * 32 * 16 * 520 bytes > 4 MiB
    big = lambda t: t.expand(B, *t.shape[1:]).contiguous()
    out = torch.zeros((B, 1, 32, 128), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((B, 32), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.InfLLMv2Error, match="unsupported"):
        binding.sparse_attn_decode_noalloc(prm, big(qd), big(kd), big(vd), sl.expand(B).contiguous(), T, big(idx),
                                           out, lse)
