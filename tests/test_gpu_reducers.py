"""GPU parity of apbv_compress_kv_reduced: the max and softmax-sum reductions of the score matrix of Alg. 1.

The kernels accumulate bf16 products in fp32 on the matrix cores, the oracle in fp64, so scores are compared within a
tolerance and the selection -- a decision floating point takes -- is checked by what is unique: the selected set and
its order must be right for every pair of keys whose oracle scores differ by more than the tolerance, the order must
be exact with respect to the scores the kernel itself reports, and the gathered rows must be bit copies."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2601_21444_amd as apbv
from paper_2601_21444_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def host_bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def rand_bits(rng, shape, scale=1.0):
    return wl.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def check_selection(idx, s_ref, s_gpu, l_p, tol):
    """idx [l_p] against oracle scores s_ref [L] and the kernel's own scores s_gpu [L]."""
    L = s_ref.shape[0]
    assert idx.shape == (l_p,) and len(set(idx.tolist())) == l_p and idx.min() >= 0 and idx.max() < L
    # exact with respect to the scores the kernel ranked (score descending, index ascending)
    np.testing.assert_array_equal(idx, np.argsort(-(s_gpu + 0.0), kind="stable")[:l_p])
    # right with respect to the oracle wherever the oracle's scores are separated by more than the tolerance
    sel = s_ref[idx]
    assert np.all(sel[:-1] >= sel[1:] - 2 * tol)
    rest = np.ones(L, dtype=bool)
    rest[idx] = False
    if rest.any():
        assert sel.min() >= s_ref[rest].max() - 2 * tol
    want = oracle.arg_top(s_ref, l_p)
    gaps_ok = np.ones(l_p, dtype=bool)            # positions whose oracle score is isolated from both neighbours
    sw = s_ref[np.argsort(-s_ref, kind="stable")]
    for i in range(l_p):
        if i > 0 and sw[i - 1] - sw[i] <= 2 * tol:
            gaps_ok[i] = False
        if i + 1 < L and sw[i] - sw[i + 1] <= 2 * tol:
            gaps_ok[i] = False
    np.testing.assert_array_equal(idx[gaps_ok], want[gaps_ok])
    return int(gaps_ok.sum())


# Score tolerances relative to the largest score of the head.  A logit is a sum of 64..128 products that are exact
# in fp32, accumulated in fp32: its error is a few 2^-24 of the accumulated magnitude (observed <= 2e-7 of the
# largest score).  The softmax mass adds the fp32 exp2 and the row normalisers and sums up to 512 probabilities
# (observed <= 1e-6).
TOL_MAX = 1e-6
TOL_MASS = 5e-6

CASES = [
    # hq, hkv, d, n_q, L, l_p
    (4, 2, 128, 8, 512, 32),          # the tiny configuration's shape
    (6, 2, 64, 5, 777, 100),          # 15 rows (a ragged row block), ragged key tail
    (28, 4, 128, 64, 4096, 256),      # group of 7: 448 rows
    (2, 2, 64, 1, 33, 33),            # one row per head, everything selected
    (16, 2, 128, 64, 16384, 1024),    # the 128K configuration's block: 512 rows
]


@pytest.mark.parametrize("reducer", ["max", "softmax_sum"])
@pytest.mark.parametrize("hq,hkv,d,n_q,L,l_p", CASES)
def test_reduced_compress_matches_oracle(reducer, hq, hkv, d, n_q, L, l_p):
    rng = np.random.default_rng((51, hq, n_q, L))
    qp, k, v = rand_bits(rng, (n_q, hq, d)), rand_bits(rng, (L, hkv, d)), rand_bits(rng, (L, hkv, d))
    scale = 1.0 / math.sqrt(d)
    print(f"reduced compress case {reducer} hq={hq} hkv={hkv} d={d} n_q={n_q} L={L} l_p={l_p}", flush=True)
    idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(qp), dev(k), dev(v), l_p, reducer=reducer, softmax_scale=scale,
                                             return_scores=True)
    torch.cuda.synchronize()
    idx, s = idx.cpu().numpy(), s.cpu().numpy()
    if reducer == "max":
        s_ref = oracle.importance_scores_max(qp, k)
        tol = TOL_MAX * np.abs(s_ref).max()
    else:
        s_ref = oracle.importance_scores_softmax_sum(qp, k, scale)
        tol = TOL_MASS * np.abs(s_ref).max()
        np.testing.assert_allclose(s.sum(axis=1), n_q * (hq // hkv), rtol=1e-4)      # every row's mass is one
    err = np.abs(s - s_ref).max()
    print(f"  scores: max abs err {err:.3e} (tolerance {tol:.3e})", flush=True)
    assert err <= tol
    k_c, v_c = host_bits(k_c), host_bits(v_c)
    for h in range(hkv):
        n_exact = check_selection(idx[h], s_ref[h], s[h], l_p, tol)
        print(f"  head {h}: {n_exact}/{l_p} positions pinned exactly", flush=True)
        np.testing.assert_array_equal(k_c[:, h], k[idx[h], h])
        np.testing.assert_array_equal(v_c[:, h], v[idx[h], h])


def test_reduced_entry_with_sum_is_the_plain_call():
    rng = np.random.default_rng(52)
    qp, k, v = rand_bits(rng, (8, 4, 128)), rand_bits(rng, (1000, 2, 128)), rand_bits(rng, (1000, 2, 128))
    lib = apbv.load_library()
    qv, kv, vv = (apbv.tensor_view(dev(x))[0] for x in (qp, k, v))
    dq, dk, dv_ = dev(qp), dev(k), dev(v)
    qv, kv, vv = apbv.tensor_view(dq)[0], apbv.tensor_view(dk)[0], apbv.tensor_view(dv_)[0]
    a = apbv.apbv_compress_kv(dq, dk, dv_, 77, return_scores=True)
    idx = torch.empty((1, 2, 77), dtype=torch.int32, device="cuda")
    kc = torch.empty((1, 77, 2, 128), dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    sc = torch.empty((1, 2, 1000), dtype=torch.float64, device="cuda")
    ws = torch.empty(apbv.apbv_compress_reduced_workspace_bytes("sum", 1, 4, 2, 128, 8, 1000, 77), dtype=torch.uint8, device="cuda")
    st = lib.apbv_compress_kv_reduced(0, 0.0, 1, 4, 2, 128, qv, kv, vv, 77, idx.data_ptr(), kc.data_ptr(), vc.data_ptr(),
                                      sc.data_ptr(), ws.data_ptr(), ws.numel(), None)
    torch.cuda.synchronize()
    assert st == 0
    assert torch.equal(a[0], idx[0]) and torch.equal(a[3], sc[0])
    assert torch.equal(a[1].view(torch.int16), kc[0].view(torch.int16)) and torch.equal(a[2].view(torch.int16), vc[0].view(torch.int16))


def test_reduced_compress_batched_strided():
    rng = np.random.default_rng(53)
    B, hq, hkv, d, n_q, L, l_p = 3, 8, 2, 128, 16, 600, 50
    scale = 1.0 / math.sqrt(d)
    qp = rand_bits(rng, (B, n_q, hq, d))
    k, v = rand_bits(rng, (B, L, hkv, d)), rand_bits(rng, (B, L, hkv, d))
    k_wide = torch.zeros((B, L, hkv, d + 64), dtype=torch.bfloat16, device="cuda")
    k_wide[..., :d] = dev(k)
    for reducer in ("max", "softmax_sum"):
        idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(qp), k_wide[..., :d], dev(v), l_p, reducer=reducer,
                                                 softmax_scale=scale, return_scores=True)
        torch.cuda.synchronize()
        for b in range(B):
            s_ref = (oracle.importance_scores_max(qp[b], k[b]) if reducer == "max"
                     else oracle.importance_scores_softmax_sum(qp[b], k[b], scale))
            tol = (TOL_MAX if reducer == "max" else TOL_MASS) * np.abs(s_ref).max()
            assert np.abs(s[b].cpu().numpy() - s_ref).max() <= tol
            for h in range(hkv):
                check_selection(idx[b, h].cpu().numpy(), s_ref[h], s[b, h].cpu().numpy(), l_p, tol)
                np.testing.assert_array_equal(host_bits(k_c[b])[:, h], k[b][idx[b, h].cpu().numpy(), h])


def test_softmax_mass_with_larger_statistics_chunks():
    """A large batch makes the statistics pass take more keys per workgroup (512 to 4096 instead of 256, a ragged last
    chunk included): every item of the batch must still match the oracle of its own data."""
    rng = np.random.default_rng(54)
    items, B, hq, hkv, d, n_q, L, l_p = 3, 200, 4, 2, 128, 30, 2500, 64       # 60 rows per head: one row group
    scale = 1.0 / math.sqrt(d)
    qp = rand_bits(rng, (items, n_q, hq, d))
    k, v = rand_bits(rng, (items, L, hkv, d)), rand_bits(rng, (items, L, hkv, d))
    pick = np.arange(B) % items
    idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(qp[pick]), dev(k[pick]), dev(v[pick]), l_p, reducer="softmax_sum",
                                             softmax_scale=scale, return_scores=True)
    torch.cuda.synchronize()
    idx, s, k_c = idx.cpu().numpy(), s.cpu().numpy(), host_bits(k_c)
    refs = [oracle.importance_scores_softmax_sum(qp[i], k[i], scale) for i in range(items)]
    for b in range(B):
        i = int(pick[b])
        tol = TOL_MASS * np.abs(refs[i]).max()
        assert np.abs(s[b] - refs[i]).max() <= tol, f"item {b}"
        np.testing.assert_allclose(s[b].sum(axis=1), n_q * (hq // hkv), rtol=1e-4)
        if b < 2 * items or b >= B - items:              # the full selection check on the first and last items
            for h in range(hkv):
                check_selection(idx[b, h], refs[i][h], s[b, h], l_p, tol)
                np.testing.assert_array_equal(k_c[b][:, h], k[i][idx[b, h], h])
