"""Seeded random-shape sweep of every attention entry point against the fp64 oracle: ragged lengths around the
tile sizes (64-key tiles, 64- and 256-row workgroups), empty segments, both head dimensions, strided views."""
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


def rand_bits(rng, shape):
    return wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def pick_len(rng, choices=(0, 1, 31, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 640)):
    return int(rng.choice(choices))


def check(out_gpu, ref, what):
    diff = np.abs(out_gpu - ref)
    assert np.all(np.isfinite(out_gpu)), what
    assert diff.max() <= 2e-2 and diff.mean() / np.abs(ref).mean() <= 5e-3, \
        f"{what}: max_abs={diff.max():.3e} mean_rel={diff.mean() / np.abs(ref).mean():.3e}"


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_all_attention_entry_points(seed):
    rng = np.random.default_rng((71, seed))
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    hq = hkv * int(rng.choice([1, 2, 4, 7]))
    scale = 1.0 / math.sqrt(d)
    L = max(pick_len(rng), 1)
    l_a, n_p = pick_len(rng), pick_len(rng)
    causal = bool(rng.integers(0, 2)) or (l_a + n_p == 0)
    n_l = L if causal else 0
    q = rand_bits(rng, (L, hq, d))
    ka, va, kp, vp, kl, vl = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_p, n_p, n_l, n_l))
    print(f"random shape seed={seed}: hq={hq} hkv={hkv} d={d} L={L} l_a={l_a} n_p={n_p} causal={causal}", flush=True)
    ref, lse_r = oracle.host_attention(q, ka, va, kp, vp, kl, vl, scale)
    # passing keys as a strided view (rows padded), everything else dense
    kp_wide = torch.zeros((n_p, hkv, d + 8), dtype=torch.bfloat16, device="cuda")
    kp_wide[..., :d] = dev(kp)
    args = [dev(q), dev(ka), dev(va), kp_wide[..., :d], dev(vp), dev(kl), dev(vl)]

    out, lse = apbv.apbv_host_attention(*args, scale, return_lse=True)
    torch.cuda.synchronize()
    check(to_f64(out), ref, "host_attention")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)

    n_splits = int(rng.choice([0, 2, 3, 7]))
    out_s, lse_s = apbv.apbv_query_attention(*args, scale, n_splits=n_splits, return_lse=True)
    torch.cuda.synchronize()
    check(to_f64(out_s), ref, f"query_attention n_splits={n_splits}")
    np.testing.assert_allclose(lse_s.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)

    if causal:
        # the same problem twice in a group with a second, different one in between
        L2 = max(pick_len(rng), 1)
        other = [rand_bits(rng, (L2, hq, d))] + [rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, 0, 0, L2, L2)]
        res = apbv.apbv_host_attention_group([tuple(args), tuple(dev(x) for x in other), tuple(args)], scale)
        torch.cuda.synchronize()
        assert torch.equal(res[0].view(torch.int16), out.view(torch.int16))
        assert torch.equal(res[2].view(torch.int16), out.view(torch.int16))
        ref2, _ = oracle.host_attention(*other, scale)
        check(to_f64(res[1]), ref2, "group, second problem")


@pytest.mark.parametrize("seed", range(8))
def test_random_mid_size_shapes_through_the_pipelined_rounds(seed):
    """Blocks of several query tiles whose key loops run tens of four-tile rounds: segment boundaries that fall inside
    a round, inside a tile, or exactly between rounds (every fifth case is aligned throughout), both head dimensions,
    group sizes 1 / 2 / 7; plain, key-split and grouped launches."""
    rng = np.random.default_rng((75, seed))
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 4]))
    hq = hkv * int(rng.choice([1, 2, 7]))
    L = int(rng.integers(600, 3000))
    l_a = int(rng.choice([0, 32, 100, 1024, 2047, 2048, 1500]))
    n_p = int(rng.choice([0, 96, 512, 1000, 3072, 3583]))
    if seed % 5 == 0:
        L, l_a, n_p = (L // 256) * 256, (l_a // 128) * 128, (n_p // 128) * 128
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (L, hq, d))
    ka, va, kp, vp, kl, vl = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_p, n_p, L, L))
    print(f"mid-size shape seed={seed}: hq={hq} hkv={hkv} d={d} L={L} l_a={l_a} n_p={n_p}", flush=True)
    ref, lse_r = oracle.host_attention(q, ka, va, kp, vp, kl, vl, scale)
    args = [dev(x) for x in (q, ka, va, kp, vp, kl, vl)]
    out, lse = apbv.apbv_host_attention(*args, scale, return_lse=True)
    out_s, lse_s = apbv.apbv_query_attention(*args, scale, n_splits=int(rng.choice([2, 5, 9])), return_lse=True)
    res = apbv.apbv_host_attention_group([tuple(args), tuple(args)], scale)
    torch.cuda.synchronize()
    check(to_f64(out), ref, "host_attention")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)
    check(to_f64(out_s), ref, "query_attention")
    np.testing.assert_allclose(lse_s.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)
    assert torch.equal(res[0].view(torch.int16), out.view(torch.int16))
    assert torch.equal(res[1].view(torch.int16), out.view(torch.int16))


@pytest.mark.parametrize("batch,hkv,group", [(4, 2, 2), (3, 2, 4), (5, 1, 3), (8, 2, 1), (2, 4, 7), (1, 8, 2), (9, 3, 2)])
def test_attention_every_way_of_dealing_items_to_the_xcds(batch, hkv, group):
    """Work items are dealt to the eight XCDs in rows of eight, odd rows in the opposite direction in groups of
    batch * Hkv XCDs where that divides eight, item by item otherwise, unchanged where it is a multiple of eight:
    every (batch, Hkv) class of that rule, over several query tiles, every item against the oracle, and the key-split
    launch (whose item count is multiplied by the number of key ranges) against the unsplit one."""
    rng = np.random.default_rng((74, batch, hkv, group))
    d, L, l_a, n_p = 64, 700, 96, 160                      # three 256-row query tiles per head
    hq = hkv * group
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (batch, L, hq, d))
    ka, va, kp, vp, kl, vl = (rand_bits(rng, (batch, n, hkv, d)) for n in (l_a, l_a, n_p, n_p, L, L))
    args = [dev(x) for x in (q, ka, va, kp, vp, kl, vl)]
    print(f"dealing: batch={batch} hkv={hkv} group={group}", flush=True)
    out, lse = apbv.apbv_host_attention(*args, scale, return_lse=True)
    out_s = apbv.apbv_query_attention(*args, scale, n_splits=3)
    torch.cuda.synchronize()
    for b in range(batch):
        ref, lse_r = oracle.host_attention(q[b], ka[b], va[b], kp[b], vp[b], kl[b], vl[b], scale)
        check(to_f64(out[b]), ref, f"item {b}")
        check(to_f64(out_s[b]), ref, f"item {b}, key split")
        np.testing.assert_allclose(lse[b].cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)


@pytest.mark.parametrize("seed", range(10))
def test_random_shapes_compress_bit_exact(seed):
    """Seeded random shapes through apbv_compress_kv: ragged block lengths around the kernels' row groupings, every
    l_p from 0 to L, both head dimensions, quantised keys (many exact ties) in half of the cases."""
    rng = np.random.default_rng((72, seed))
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 4]))
    hq = hkv * int(rng.choice([1, 3, 8]))
    n_q = int(rng.choice([1, 2, 7, 64, 130]))
    L = int(rng.choice([1, 2, 63, 64, 65, 255, 1000, 4097, 20000]))
    l_p = int(rng.choice([0, 1, L // 3, L - 1, L])) if L > 1 else int(rng.choice([0, 1]))
    l_p = max(0, min(l_p, L))
    qp = rand_bits(rng, (n_q, hq, d))
    if seed % 2:
        k = wl.f32_to_bf16_bits(rng.integers(-2, 3, size=(L, hkv, d)).astype(np.float32))     # few distinct scores
    else:
        k = rand_bits(rng, (L, hkv, d))
    v = rand_bits(rng, (L, hkv, d))
    print(f"random compress seed={seed}: hq={hq} hkv={hkv} d={d} n_q={n_q} L={L} l_p={l_p}", flush=True)
    idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(qp), dev(k), dev(v), l_p, return_scores=True)
    torch.cuda.synchronize()
    idx_r, kc_r, vc_r, s_r = oracle.compress_kv(qp, k, v, l_p)
    np.testing.assert_allclose(s.cpu().numpy(), s_r, rtol=1e-12, atol=1e-9)
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_r)
    bits_of = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(bits_of(k_c), kc_r)
    np.testing.assert_array_equal(bits_of(v_c), vc_r)


@pytest.mark.parametrize("d,hkv,group,n_q", [(128, 2, 8, 64), (64, 4, 2, 130), (128, 1, 3, 5)])
def test_compress_is_the_same_at_every_batch_size(d, hkv, group, n_q):
    """The pooled query is summed over a number of row ranges that depends on the batch size (few pooled queries:
    up to eight workgroups each; many: one or two, 1024 threads wide).  The addends are bf16 and the sums fp64, so
    with ordinary data every partition gives the same bits: an item must get identical scores and indices alone and
    inside batches of 3, 40 and 300, and every item of a batch must match the oracle."""
    rng = np.random.default_rng((73, d, hkv))
    hq, L, l_p = hkv * group, 2100, 300
    items = 4                                                   # distinct items, repeated to fill the larger batches
    qp = rand_bits(rng, (items, n_q, hq, d))
    k = rand_bits(rng, (items, L, hkv, d))
    v = rand_bits(rng, (items, L, hkv, d))
    ref = [oracle.compress_kv(qp[i], k[i], v[i], l_p) for i in range(items)]
    singles = []
    for i in range(items):
        idx, _, _, sc = apbv.apbv_compress_kv(dev(qp[i]), dev(k[i]), dev(v[i]), l_p, return_scores=True)
        np.testing.assert_array_equal(idx.cpu().numpy(), ref[i][0])
        singles.append((idx.cpu().numpy(), sc.cpu().numpy()))
    for batch in (3, 40, 300):
        pick = np.arange(batch) % items
        print(f"batch invariance: d={d} hkv={hkv} group={group} n_q={n_q} batch={batch}", flush=True)
        idx, k_c, v_c, sc = apbv.apbv_compress_kv(dev(qp[pick]), dev(k[pick]), dev(v[pick]), l_p, return_scores=True)
        torch.cuda.synchronize()
        idx, sc = idx.cpu().numpy(), sc.cpu().numpy()
        bits_of = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        k_c, v_c = bits_of(k_c), bits_of(v_c)
        for b in range(batch):
            i = int(pick[b])
            assert np.array_equal(sc[b].view(np.uint64), singles[i][1].view(np.uint64)), f"scores of item {b} differ from the single call"
            np.testing.assert_array_equal(idx[b], singles[i][0])
            np.testing.assert_array_equal(k_c[b], ref[i][1])
            np.testing.assert_array_equal(v_c[b], ref[i][2])


@pytest.mark.parametrize("gain", [8.0, 40.0])
def test_attention_with_peaked_logits(gain):
    """Queries scaled up so that the softmax is nearly one-hot and the running maximum jumps by far more than the
    lazy-rescale threshold from tile to tile (scaled logits up to several hundred): no overflow, same tolerances."""
    rng = np.random.default_rng((73, int(gain)))
    hq, hkv, d, L, l_a, n_p = 4, 2, 128, 300, 200, 500
    scale = 1.0 / math.sqrt(d)
    q = wl.f32_to_bf16_bits((rng.standard_normal((L, hq, d)) * gain).astype(np.float32))
    ka, va, kp, vp, k, v = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_p, n_p, L, L))
    # ascending key norms along the key axis make the maximum grow again and again
    grow = np.linspace(0.2, 2.0, n_p, dtype=np.float32)[:, None, None]
    kp = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(kp) * grow)
    out, lse = apbv.apbv_host_attention(*[dev(x) for x in (q, ka, va, kp, vp, k, v)], scale, return_lse=True)
    torch.cuda.synchronize()
    ref, lse_r = oracle.host_attention(q, ka, va, kp, vp, k, v, scale)
    print(f"peaked logits gain={gain}: lse range {lse_r.min():.1f} .. {lse_r.max():.1f}", flush=True)
    check(to_f64(out), ref, f"peaked logits x{gain}")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, rtol=2e-5, atol=2e-3)
