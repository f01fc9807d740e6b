"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same seeded inputs.

Bars: top-l_p indices and gathered rows bit-exact; attention within max-abs 2e-2 and mean-rel 5e-3
(mean|diff| / mean|ref| over the tensor), bf16 inputs, fp32 accumulation."""
import math
import zlib

import numpy as np
import pytest
import torch

import oracle
import paper_2601_21444_amd as apbv
from paper_2601_21444_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_ABS = 2e-2
MEAN_REL = 5e-3


def dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (numpy uint16) -> bfloat16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return wl.bf16_bits_to_f32(host_bits(t)).astype(np.float64)


def check_attention(out_gpu: np.ndarray, ref: np.ndarray, what: str):
    diff = np.abs(out_gpu - ref)
    max_abs = float(diff.max())
    mean_rel = float(diff.mean() / np.abs(ref).mean())
    print(f"{what}: max_abs={max_abs:.3e} mean_rel={mean_rel:.3e}", flush=True)
    assert np.all(np.isfinite(out_gpu)), what
    assert max_abs <= MAX_ABS, (what, max_abs)
    assert mean_rel <= MEAN_REL, (what, mean_rel)


def check_attention_quiet(out_gpu: np.ndarray, ref: np.ndarray, what: str):
    diff = np.abs(out_gpu - ref)
    assert float(diff.max()) <= MAX_ABS, (what, float(diff.max()))
    assert float(diff.mean() / np.abs(ref).mean()) <= MEAN_REL, what


def oracle_passing(x):
    c = x.cfg
    return oracle.make_passing_block(x.q_probe, x.k_prev, x.v_prev, c.l_p, c.n_kv_heads, c.head_dim)


def run_attention(x, k_p, v_p, lse=False):
    scale = 1.0 / math.sqrt(x.cfg.head_dim)
    res = apbv.apbv_host_attention(dev(x.q), dev(x.k_anchor), dev(x.v_anchor), dev(k_p), dev(v_p), dev(x.k), dev(x.v),
                                   scale, return_lse=lse)
    torch.cuda.synchronize()
    return res, scale


# ------------------------------------------------------------------------------------------ compress

def check_compress(cfg, x=None, tamper=None, l_p=None):
    x = x or wl.generate(cfg)
    cfg = x.cfg
    if tamper:
        tamper(x)
    l_p = cfg.l_p if l_p is None else l_p
    print(f"compress {cfg.name}: L={cfg.L} Hkv={cfg.n_kv_heads} d={cfg.head_dim} l_p={l_p}", flush=True)
    idx_r, kc_r, vc_r, s_r = oracle.compress_kv(x.q_probe, x.k, x.v, l_p)
    idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(x.q_probe), dev(x.k), dev(x.v), l_p, return_scores=True)
    torch.cuda.synchronize()
    s = s.cpu().numpy()
    np.testing.assert_allclose(s, s_r, rtol=1e-13, atol=1e-12 * max(1.0, float(np.abs(s_r).max())))
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_r)
    np.testing.assert_array_equal(host_bits(k_c), kc_r)
    np.testing.assert_array_equal(host_bits(v_c), vc_r)
    return x, idx_r, s_r


def test_compress_tiny_config():
    check_compress("tiny")


@pytest.mark.parametrize("name", ["3b-8k", "3b-128k", "7b-frames", "imbalance-h1", "imbalance-h8", "imbalance-h15"])
def test_compress_full_size_configs(name):
    x, idx_r, s_r = check_compress(name)
    # report how close the ranking is to a flip: smallest gap between neighbours in the top l_p + 1
    for h in range(x.cfg.n_kv_heads):
        top = np.sort(s_r[h])[::-1][: x.cfg.l_p + 1]
        print(f"  head {h}: min adjacent gap {np.min(-np.diff(top)):.3e}, score std {s_r[h].std():.3e}", flush=True)


@pytest.mark.parametrize("hq,hkv,d,n_q,L,l_p", [
    (2, 1, 64, 8, 77, 5), (4, 4, 128, 3, 1000, 1000), (6, 2, 128, 16, 4099, 257), (7, 1, 64, 1, 64, 64),
    (8, 2, 128, 64, 16384, 16384), (2, 2, 64, 5, 300, 0), (4, 1, 128, 7, 1, 1), (2, 1, 128, 4, 9000, 8193),
])
def test_compress_shape_sweep(hq, hkv, d, n_q, L, l_p):
    check_compress(wl.custom(f"sweep{L}", (7, L, l_p), hq, hkv, d, n_q, 0, 0, 0, l_p, L))


def test_compress_planted_ties_straddling_the_cut():
    cfg = wl.custom("ties", 31, 4, 2, 128, 8, 0, 0, 0, 64, 2048)

    def tamper(x):
        _, _, _, s = oracle.compress_kv(x.q_probe, x.k, x.v, cfg.l_p)
        for h in range(2):
            order = np.argsort(-s[h], kind="stable")
            src = order[cfg.l_p - 2]                      # a key just inside the cut
            for j in (5, 700, 1500, 2047, 64, 1023):      # six more copies: ties straddle the cut
                x.k[j, h] = x.k[src, h]
    x, idx_r, s_r = check_compress(cfg, tamper=tamper)
    for h in range(2):
        top = s_r[h][idx_r[h]]
        assert np.sum(s_r[h] == top[-1]) > np.sum(top == top[-1]) >= 2      # the cut really splits a tie group


def test_compress_all_equal_scores_and_signed_zero():
    cfg = wl.custom("zeros", 1, 2, 1, 64, 4, 0, 0, 0, 10, 333)

    def tamper(x):
        x.k[:] = 0
        x.k[1::2] = 0x8000          # -0.0 keys: scores +0 / -0 alternate; all tie
    x, idx_r, _ = check_compress(cfg, tamper=tamper)
    assert idx_r[0].tolist() == list(range(10))


def test_compress_heavy_duplicates_force_the_exact_radix_path():
    """8000 copies of one key row hold the cut: the value-bucket fast path cannot fit its candidates and the
    radix path must break the tie by index; a second case puts the cut just above the cluster."""
    for l_p, n_hot in ((100, 30), (100, 300)):
        cfg = wl.custom("dups", (41, n_hot), 4, 2, 128, 8, 0, 0, 0, l_p, 9000)

        def tamper(x, n_hot=n_hot):
            rng = np.random.default_rng(n_hot)
            keep = rng.choice(9000, size=n_hot, replace=False)         # rows that stay random
            _, _, _, s = oracle.compress_kv(x.q_probe, x.k, x.v, 1)
            for h in range(2):
                src = int(np.argsort(s[h])[4500])                        # a median-score row
                row = x.k[src, h].copy()
                mask = np.ones(9000, dtype=bool)
                mask[keep] = False
                x.k[mask, h] = row
        check_compress(cfg, tamper=tamper)


def test_compress_batched_and_strided_views():
    cfg = wl.custom("b", 12, 8, 2, 128, 16, 0, 0, 0, 100, 1500)
    xs = [wl.generate(wl.custom("b", (12, i), 8, 2, 128, 16, 0, 0, 0, 100, 1500)) for i in range(3)]
    # K and V interleaved in one buffer [batch, L, 2, Hkv, d]: token stride 2*Hkv*d
    kvbuf = torch.stack([torch.stack([dev(x.k), dev(x.v)], dim=1) for x in xs])        # [3, L, 2, Hkv, d]
    qp = torch.stack([dev(x.q_probe) for x in xs])
    idx, k_c, v_c = apbv.apbv_compress_kv(qp, kvbuf[:, :, 0], kvbuf[:, :, 1], cfg.l_p)
    torch.cuda.synchronize()
    for i, x in enumerate(xs):
        idx_r, kc_r, vc_r, _ = oracle.compress_kv(x.q_probe, x.k, x.v, cfg.l_p)
        np.testing.assert_array_equal(idx[i].cpu().numpy(), idx_r)
        np.testing.assert_array_equal(host_bits(k_c[i]), kc_r)
        np.testing.assert_array_equal(host_bits(v_c[i]), vc_r)


# ------------------------------------------------------------------------------------------ attention

def test_attention_tiny_config_full():
    x = wl.generate("tiny")
    k_p, v_p = oracle_passing(x)
    (out, lse), scale = run_attention(x, k_p, v_p, lse=True)
    ref, lse_r = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, k_p, v_p, x.k, x.v, scale)
    check_attention(to_f64(out), ref, "tiny")
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)


@pytest.mark.parametrize("hq,hkv,d,l_a,P,l_p,L", [
    (2, 1, 64, 0, 0, 0, 300),         # plain causal attention, ragged
    (4, 2, 128, 0, 0, 0, 129),
    (8, 1, 128, 37, 2, 19, 257),      # nothing a multiple of the tile
    (7, 1, 128, 64, 1, 100, 511),     # GQA 7
    (4, 4, 64, 5, 3, 33, 64),         # GQA 1
    (16, 2, 128, 128, 0, 0, 384),     # anchor only
    (2, 2, 128, 0, 3, 64, 1),         # a single query row
    (6, 3, 64, 1, 1, 1, 1000),
])
def test_attention_shape_sweep(hq, hkv, d, l_a, P, l_p, L):
    cfg = wl.custom(f"att{L}", (9, L, l_a), hq, hkv, d, 4, l_a, P, max(l_p, 1) * 3, l_p, L)
    x = wl.generate(cfg)
    k_p, v_p = oracle_passing(x)
    (out, lse), scale = run_attention(x, k_p, v_p, lse=True)
    ref, lse_r = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, k_p, v_p, x.k, x.v, scale)
    check_attention(to_f64(out), ref, cfg.name)
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)


def sample_rows(L: int, name: str, per_slice: int = 1) -> np.ndarray:
    """A stratified sample of query rows: `per_slice` random rows from EVERY 32-row slice (one wave's rows; eight
    slices make a 256-row query tile), so no query tile and no wave of any tile goes uncompared, plus the first/last
    rows and the rows around tile edges.  The random choice is seeded by the configuration's name."""
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, L // 2 - 1, L // 2, L - 257, L - 256, L - 130, L - 129,
             L - 128, L - 65, L - 2, L - 1]
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    rows = set(r for r in fixed if 0 <= r < L)
    for lo in range(0, L, 32):
        hi = min(lo + 32, L)
        rows.update(rng.integers(lo, hi, size=per_slice).tolist())
    return np.array(sorted(rows), dtype=np.int64)


def check_convex_and_finite(x, v_p, full):
    """Properties that hold for every row at any size: finite, inside the range of V (softmax is convex)."""
    assert np.all(np.isfinite(full))
    segs = [a for a in (x.v_anchor, v_p, x.v) if a.size]
    vmax = max(float(wl.bf16_bits_to_f32(a).max()) for a in segs)
    vmin = min(float(wl.bf16_bits_to_f32(a).min()) for a in segs)
    assert full.max() <= vmax * 1.01 and full.min() >= vmin * 1.01


def test_attention_headline_config_every_row():
    """The headline configuration (16K local block, Eq. 4) in the launch bench.py times: EVERY output element
    (16384 rows x 16 heads x 128) and every log-sum-exp against the oracle, to the spec bars."""
    x = wl.generate(wl.HEADLINE)
    cfg = x.cfg
    print(f"attention {cfg.name} (all rows): L={cfg.L} S_kv={cfg.s_kv} Hq={cfg.n_q_heads}", flush=True)
    k_p, v_p = oracle_passing(x)
    (out, lse), scale = run_attention(x, k_p, v_p, lse=True)
    got = to_f64(out)
    lse_g = lse.cpu().numpy().astype(np.float64)
    worst_abs, sum_diff, sum_ref = 0.0, 0.0, 0.0
    step = 2048
    for lo in range(0, cfg.L, step):
        rows = np.arange(lo, min(lo + step, cfg.L), dtype=np.int64)
        ref, lse_r = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, k_p, v_p, x.k, x.v, scale, rows=rows, chunk=256)
        diff = np.abs(got[rows] - ref)
        # each 256-row query tile also meets the bars on its own (a bad tile cannot hide in the global mean)
        for t in range(0, rows.shape[0], 256):
            check_attention_quiet(got[rows[t: t + 256]], ref[t: t + 256], f"{cfg.name} rows {lo + t}..")
        worst_abs = max(worst_abs, float(diff.max()))
        sum_diff += float(diff.sum())
        sum_ref += float(np.abs(ref).sum())
        np.testing.assert_allclose(lse_g[:, rows], lse_r, atol=2e-3, rtol=0)
        print(f"  rows {lo}..{rows[-1]}: max_abs so far {worst_abs:.3e}", flush=True)
    mean_rel = sum_diff / sum_ref
    print(f"{cfg.name} all rows: max_abs={worst_abs:.3e} mean_rel={mean_rel:.3e}", flush=True)
    assert worst_abs <= MAX_ABS and mean_rel <= MEAN_REL
    check_convex_and_finite(x, v_p, got)


@pytest.mark.parametrize("name", ["3b-8k", "7b-frames", "imbalance-h1", "imbalance-h8", "imbalance-h15"])
def test_attention_full_size_configs_sampled_rows(name):
    """Full-size launch exactly as bench.py times it; the oracle evaluates complete rows for a stratified sample that
    touches every 32-row wave slice of every query tile."""
    x = wl.generate(name)
    cfg = x.cfg
    print(f"attention {name}: L={cfg.L} S_kv={cfg.s_kv} Hq={cfg.n_q_heads}", flush=True)
    k_p, v_p = oracle_passing(x)
    (out, lse), scale = run_attention(x, k_p, v_p, lse=True)
    rows = sample_rows(cfg.L, name)
    assert np.unique(rows // 32).shape[0] == (cfg.L + 31) // 32
    ref, lse_r = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, k_p, v_p, x.k, x.v, scale, rows=rows, chunk=64)
    full = to_f64(out)
    check_attention(full[rows], ref, name)
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64)[:, rows], lse_r, atol=2e-3, rtol=0)
    check_convex_and_finite(x, v_p, full)


def needle_key(qrow, d):
    return (8.0 * qrow / np.linalg.norm(qrow) * math.sqrt(d)).astype(np.float32)


def test_attention_mask_needles_on_gpu():
    """An overwhelming key planted at a masked position must not move the row; planted at each visible
    boundary position it must become the row's output.  Rows chosen at tile and wave edges."""
    cfg = wl.custom("needle", 77, 4, 2, 128, 4, 70, 2, 200, 45, 300)
    x = wl.generate(cfg)
    k_p, v_p = oracle_passing(x)
    scale = 1.0
    qf = oracle.bf16_bits_to_f64(x.q)
    base = apbv.apbv_host_attention(dev(x.q), dev(x.k_anchor), dev(x.v_anchor), dev(k_p), dev(v_p), dev(x.k), dev(x.v), scale)
    base = to_f64(base)
    h, kv = 3, 1
    for i in (0, 31, 32, 63, 64, 127, 128, 200, 298):
        nk = wl.f32_to_bf16_bits(needle_key(qf[i, h], cfg.head_dim))
        # masked: local key i+1
        k2 = x.k.copy()
        k2[i + 1, kv] = nk
        o = to_f64(apbv.apbv_host_attention(dev(x.q), dev(x.k_anchor), dev(x.v_anchor), dev(k_p), dev(v_p), dev(k2), dev(x.v), scale))
        np.testing.assert_array_equal(o[i, h], base[i, h])
        # visible boundaries
        for seg, pos in (("l", i), ("l", 0), ("a", cfg.l_a - 1), ("a", 0), ("p", 0), ("p", k_p.shape[0] - 1)):
            ka, kp_, kl = x.k_anchor.copy(), k_p.copy(), x.k.copy()
            tgt, vsrc = {"a": (ka, x.v_anchor), "p": (kp_, v_p), "l": (kl, x.v)}[seg]
            tgt[pos, kv] = nk
            o = to_f64(apbv.apbv_host_attention(dev(x.q), dev(ka), dev(x.v_anchor), dev(kp_), dev(v_p), dev(kl), dev(x.v), scale))
            np.testing.assert_allclose(o[i, h], oracle.bf16_bits_to_f64(vsrc)[pos, kv], atol=1e-6, err_msg=f"{i} {seg} {pos}")


def test_attention_uncompressed_passing_equals_dense_on_gpu():
    """l_p = block length: GPU compress + GPU attention must reproduce dense attention over the full
    preceding blocks (whole hot path end to end, oracle only as the dense reference)."""
    cfg = wl.custom("nocomp", 15, 4, 2, 128, 8, 32, 2, 256, 256, 320)
    x = wl.generate(cfg)
    kps, vps = [], []
    for kp, vp in zip(x.k_prev, x.v_prev):
        _, k_c, v_c = apbv.apbv_compress_kv(dev(x.q_probe), dev(kp), dev(vp), cfg.l_p)
        kps.append(k_c)
        vps.append(v_c)
    scale = 1.0 / math.sqrt(cfg.head_dim)
    out = apbv.apbv_host_attention(dev(x.q), dev(x.k_anchor), dev(x.v_anchor), torch.cat(kps), torch.cat(vps), dev(x.k), dev(x.v), scale)
    ref, _ = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, np.concatenate(x.k_prev), np.concatenate(x.v_prev), x.k, x.v, scale)
    check_attention(to_f64(out), ref, "nocomp-dense")


def test_attention_batched_strided_and_deterministic():
    cfg = wl.custom("bs", 3, 8, 2, 128, 4, 40, 1, 128, 24, 200)
    xs = [wl.generate(wl.custom("bs", (3, i), 8, 2, 128, 4, 40, 1, 128, 24, 200)) for i in range(2)]
    pas = [oracle_passing(x) for x in xs]
    scale = 1.0 / math.sqrt(128)
    # one concatenated KV buffer per batch item; the three segments are views into it
    kcat = torch.stack([torch.cat([dev(x.k_anchor), dev(p[0]), dev(x.k)]) for x, p in zip(xs, pas)])
    vcat = torch.stack([torch.cat([dev(x.v_anchor), dev(p[1]), dev(x.v)]) for x, p in zip(xs, pas)])
    q = torch.stack([dev(x.q) for x in xs])
    a, n = cfg.l_a, cfg.l_a + cfg.P * cfg.l_p
    args = (q, kcat[:, :a], vcat[:, :a], kcat[:, a:n], vcat[:, a:n], kcat[:, n:], vcat[:, n:], scale)
    # canaries around the output
    buf = torch.full((2 * cfg.L * 8 * 128 + 512,), -7.0, dtype=torch.bfloat16, device="cuda")
    out = buf[256:-256].view(2, cfg.L, 8, 128)
    apbv.apbv_host_attention(*args, out=out)
    out2 = apbv.apbv_host_attention(*args)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    assert torch.all(buf[:256] == -7.0) and torch.all(buf[-256:] == -7.0)
    for i, (x, p) in enumerate(zip(xs, pas)):
        ref, _ = oracle.host_attention(x.q, x.k_anchor, x.v_anchor, p[0], p[1], x.k, x.v, scale)
        check_attention(to_f64(out[i]), ref, f"batched[{i}]")


def test_errors_surface_as_exceptions():
    q = torch.zeros((64, 3, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((64, 2, 128), dtype=torch.bfloat16, device="cuda")
    e = k[:0]
    with pytest.raises(apbv.ApbvError):
        apbv.apbv_host_attention(q, e, e, e, e, k, k, 0.1)
    with pytest.raises(apbv.ApbvError):
        apbv.apbv_compress_kv(q[:4, :2], k, k, 65)
