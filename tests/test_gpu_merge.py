"""GPU parity for the query-block path of Eq. 5: partial attention without a causal segment, and the
log-sum-exp merge of partial results, against the fp64 oracle."""
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


def to_f64(t):
    return wl.bf16_bits_to_f32(t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)


def check(out_gpu, ref, what, max_abs=2e-2, mean_rel=5e-3):
    diff = np.abs(out_gpu - ref)
    print(f"{what}: max_abs={diff.max():.3e} mean_rel={diff.mean() / np.abs(ref).mean():.3e}", flush=True)
    assert np.all(np.isfinite(out_gpu))
    assert diff.max() <= max_abs and diff.mean() / np.abs(ref).mean() <= mean_rel


def rand_bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("hq,hkv,d,n_q,l_a,n_c", [(4, 2, 128, 64, 100, 700), (8, 1, 64, 7, 0, 130), (16, 2, 128, 300, 64, 0), (2, 2, 128, 1, 1, 0)])
def test_partial_attention_without_causal_segment(hq, hkv, d, n_q, l_a, n_c):
    rng = np.random.default_rng((3, n_q, n_c))
    q = rand_bits(rng, (n_q, hq, d))
    ka, va, kc, vc = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_c, n_c))
    e = np.empty((0, hkv, d), dtype=np.uint16)
    scale = 1.0 / math.sqrt(d)
    out, lse = apbv.apbv_host_attention(dev(q), dev(ka), dev(va), dev(kc), dev(vc), dev(e), dev(e), scale, return_lse=True)
    torch.cuda.synchronize()
    ref, lse_r = oracle.host_attention(q, ka, va, kc, vc, e, e, scale)
    check(to_f64(out), ref, f"partial n_q={n_q}")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)


def test_merge_matches_oracle_and_handles_empty_parts():
    rng = np.random.default_rng(9)
    n, rows, hq, d = 5, 77, 6, 128
    outs = rand_bits(rng, (n, rows, hq, d))
    lses = (rng.standard_normal((n, hq, rows)) * 3).astype(np.float32)
    lses[2] = -np.inf                       # a part that saw no key
    lses[:, 1, 5] = -np.inf                 # a row with no key anywhere
    buf = torch.full((n, rows * hq * d + 64), 3.0, dtype=torch.bfloat16, device="cuda")     # padded part stride
    parts = buf[:, : rows * hq * d].view(n, rows, hq, d)
    parts.copy_(dev(outs))
    out, lse = apbv.apbv_merge_lse(parts, torch.from_numpy(lses).cuda(), return_lse=True)
    torch.cuda.synchronize()
    ref, lse_r = oracle.merge_lse([wl.bf16_bits_to_f32(outs[i]).astype(np.float64) for i in range(n)], list(lses.astype(np.float64)))
    got = to_f64(out)
    diff = np.abs(got - ref)
    assert diff.max() <= 2e-2 and diff.mean() / np.abs(ref).mean() <= 3e-3
    assert np.all(got[5, 1] == 0)
    lse_g = lse.cpu().numpy().astype(np.float64)
    assert lse_g[1, 5] == -np.inf
    fin = np.isfinite(lse_r)
    np.testing.assert_allclose(lse_g[fin], lse_r[fin], atol=1e-5)


def test_query_block_attention_end_to_end():
    """Eq. 5 on one GPU: H hosts each attend the query block to their anchor slice and context block (no causal
    segment), the last one also to the query block's own keys (causal); the merged result must equal
    attention of the query block over everything."""
    rng = np.random.default_rng(12)
    H, hq, hkv, d, n_q, l_a, l_b = 4, 8, 2, 128, 64, 256, 1024
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (n_q, hq, d))
    ka, va = rand_bits(rng, (l_a, hkv, d)), rand_bits(rng, (l_a, hkv, d))
    kc = [rand_bits(rng, (l_b, hkv, d)) for _ in range(H)]
    vc = [rand_bits(rng, (l_b, hkv, d)) for _ in range(H)]
    kq, vq = rand_bits(rng, (n_q, hkv, d)), rand_bits(rng, (n_q, hkv, d))
    e = np.empty((0, hkv, d), dtype=np.uint16)
    sl = l_a // H
    parts_o = torch.empty((H, n_q, hq, d), dtype=torch.bfloat16, device="cuda")
    parts_l = torch.empty((H, hq, n_q), dtype=torch.float32, device="cuda")
    for h in range(H):
        own = (dev(kq), dev(vq)) if h == H - 1 else (dev(e), dev(e))
        apbv.apbv_host_attention(dev(q), dev(ka[h * sl:(h + 1) * sl]), dev(va[h * sl:(h + 1) * sl]), dev(kc[h]), dev(vc[h]),
                                 own[0], own[1], scale, out=parts_o[h:h + 1], lse_out=parts_l[h:h + 1])
    out = apbv.apbv_merge_lse(parts_o, parts_l)
    torch.cuda.synchronize()
    ref, _ = oracle.host_attention(q, ka, va, np.concatenate(kc), np.concatenate(vc), kq, vq, scale)
    check(to_f64(out), ref, "query block, merged over hosts")


# ---- key-split attention of a short query block (apbv_query_attention) ---------------------------------------------
SPLIT_CASES = [
    # hq, hkv, d, n_q, l_a, n_c, local, n_splits
    (4, 2, 128, 64, 100, 700, False, 4),       # ranges cross the anchor/passing boundary, ragged last tile
    (8, 1, 64, 7, 0, 130, False, 3),           # three tiles, one per range, the last with two keys
    (4, 4, 128, 1, 65, 0, False, 2),           # a single query; second range holds a single key
    (6, 2, 128, 300, 100, 200, True, 5),       # causal local segment: late ranges are empty for early rows
    (6, 2, 64, 300, 0, 0, True, 4),            # causal only
    (4, 2, 128, 40, 64, 3000, False, 0),       # library's choice
    (4, 2, 128, 40, 64, 3000, False, 1000),    # more ranges than tiles: clipped
]


@pytest.mark.parametrize("hq,hkv,d,n_q,l_a,n_c,local,n_splits", SPLIT_CASES)
def test_query_attention_key_split_matches_oracle(hq, hkv, d, n_q, l_a, n_c, local, n_splits):
    rng = np.random.default_rng((21, n_q, n_c, n_splits))
    q = rand_bits(rng, (n_q, hq, d))
    ka, va, kc, vc = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_c, n_c))
    n_l = n_q if local else 0
    kl, vl = rand_bits(rng, (n_l, hkv, d)), rand_bits(rng, (n_l, hkv, d))
    scale = 1.0 / math.sqrt(d)
    args = [dev(x) for x in (q, ka, va, kc, vc, kl, vl)]
    print(f"query_attention case hq={hq} d={d} n_q={n_q} keys={l_a}+{n_c}+{n_l} splits={n_splits}", flush=True)
    out, lse = apbv.apbv_query_attention(*args, scale, n_splits=n_splits, return_lse=True)
    plain, lse_p = apbv.apbv_host_attention(*args, scale, return_lse=True)
    torch.cuda.synchronize()
    ref, lse_r = oracle.host_attention(q, ka, va, kc, vc, kl, vl, scale)
    check(to_f64(out), ref, f"key split {n_splits}")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)
    # the split result differs from the unsplit kernel's by the bf16 rounding of the parts at most
    assert np.abs(to_f64(out) - to_f64(plain)).max() <= 2e-2
    # (row sums are taken over the bf16-rounded probabilities, whose rounding depends on each range's own maximum)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_p.cpu().numpy(), atol=1e-3, rtol=0)


def test_query_attention_single_range_is_the_plain_kernel():
    rng = np.random.default_rng(22)
    hq, hkv, d, n_q, n_c = 4, 2, 128, 33, 500
    q, kc, vc = rand_bits(rng, (n_q, hq, d)), rand_bits(rng, (n_c, hkv, d)), rand_bits(rng, (n_c, hkv, d))
    e = np.empty((0, hkv, d), dtype=np.uint16)
    args = [dev(x) for x in (q, e, e, kc, vc, e, e)]
    a = apbv.apbv_query_attention(*args, 0.09, n_splits=1)
    b = apbv.apbv_host_attention(*args, 0.09)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_query_attention_batched_strided_and_deterministic():
    rng = np.random.default_rng(23)
    B, hq, hkv, d, n_q, l_a, n_c = 3, 8, 2, 128, 50, 70, 900
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (B, n_q, hq, d))
    ka, va, kc, vc = (rand_bits(rng, (B, n, hkv, d)) for n in (l_a, l_a, n_c, n_c))
    e = torch.empty((B, 0, hkv, d), dtype=torch.bfloat16, device="cuda")
    kc_wide = torch.zeros((B, n_c, hkv, d + 64), dtype=torch.bfloat16, device="cuda")      # padded rows: strided view
    kc_wide[..., :d] = dev(kc)
    args = [dev(q), dev(ka), dev(va), kc_wide[..., :d], dev(vc), e, e]
    out1 = apbv.apbv_query_attention(*args, scale, n_splits=6)
    out2 = apbv.apbv_query_attention(*args, scale, n_splits=6)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    e_np = np.empty((0, hkv, d), dtype=np.uint16)
    for b in range(B):
        ref, _ = oracle.host_attention(q[b], ka[b], va[b], kc[b], vc[b], e_np, e_np, scale)
        check(to_f64(out1[b]), ref, f"batched key split, item {b}")


def test_query_attention_full_size_sampled_rows():
    """A 512-token query block of the 3B model over one host's 16K-token context block plus anchor, at the library's
    own split; sampled rows against the oracle."""
    cfg = wl.CONFIGS["3b-128k"]
    rng = np.random.default_rng(24)
    hq, hkv, d, n_q = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, 512
    l_a, n_c = cfg.l_a, cfg.L
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (n_q, hq, d))
    ka, va, kc, vc = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_c, n_c))
    e = np.empty((0, hkv, d), dtype=np.uint16)
    out = apbv.apbv_query_attention(*[dev(x) for x in (q, ka, va, kc, vc, e, e)], scale)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 255, 256, 300, 511])
    ref, _ = oracle.host_attention(q, ka, va, kc, vc, e, e, scale, rows=rows)
    check(to_f64(out)[rows], ref, "full-size query block, sampled rows")
