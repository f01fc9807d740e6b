"""GPU parity of apbv_host_attention_group: the attention problems of a physical host (both virtual hosts' context
attention, the anchor block's own causal attention; Alg. 1, Sec. 4.3) in one launch, against the fp64 oracle and
against separate apbv_host_attention calls."""
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


def make_problem(rng, hq, hkv, d, L, l_a, n_p):
    q = rand_bits(rng, (L, hq, d))
    ka, va, kp, vp, k, v = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_p, n_p, L, L))
    return (q, ka, va, kp, vp, k, v)


def check(out_gpu, ref, what, max_abs=2e-2, mean_rel=5e-3):
    diff = np.abs(out_gpu - ref)
    print(f"{what}: max_abs={diff.max():.3e} mean_rel={diff.mean() / np.abs(ref).mean():.3e}", flush=True)
    assert np.all(np.isfinite(out_gpu))
    assert diff.max() <= max_abs and diff.mean() / np.abs(ref).mean() <= mean_rel


GROUPS = [
    # (hq, hkv, d, [(L, l_a, n_p), ...])
    (4, 2, 128, [(300, 0, 0), (700, 300, 0), (700, 300, 450)]),           # anchor block + two virtual hosts
    (8, 2, 64, [(257, 10, 1000), (1, 0, 0), (513, 0, 255), (256, 256, 0)]),
    (2, 1, 128, [(100, 5, 5)]),                                             # a group of one
    (2, 2, 128, [(64 + 37 * m, 16 * m, 300 * (7 - m)) for m in range(8)]),  # the maximum of eight problems
    # KV head counts that divide eight, do not divide it, equal it (the three ways entries are dealt to the XCDs),
    # each over enough query tiles for several rows of eight entries
    (6, 3, 64, [(900, 64, 0), (1300, 64, 200)]),
    (8, 4, 64, [(1100, 0, 100), (600, 32, 0), (300, 0, 0)]),
    (8, 8, 64, [(800, 16, 16), (520, 0, 0)]),
]


@pytest.mark.parametrize("hq,hkv,d,shapes", GROUPS)
def test_group_matches_oracle_and_separate_calls(hq, hkv, d, shapes):
    rng = np.random.default_rng((31, hq, d, len(shapes)))
    scale = 1.0 / math.sqrt(d)
    probs = [make_problem(rng, hq, hkv, d, *sh) for sh in shapes]
    dprobs = []
    for pr in probs:
        L = pr[0].shape[0]
        out = torch.full((L + 2, hq, d), float("nan"), dtype=torch.bfloat16, device="cuda")   # a canary row on both sides
        dprobs.append(tuple(dev(x) for x in pr) + (out[1:L + 1],))
    print(f"group case hq={hq} hkv={hkv} d={d} shapes={shapes}", flush=True)
    res = apbv.apbv_host_attention_group(dprobs, scale, return_lse=True)
    torch.cuda.synchronize()
    for m, (pr, dp, (out, lse)) in enumerate(zip(probs, dprobs, res)):
        whole = dp[7]._base if dp[7]._base is not None else None
        ref, lse_r = oracle.host_attention(*pr, scale)
        check(to_f64(out), ref, f"problem {m} {shapes[m]}")
        np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)
        plain, lse_p = apbv.apbv_host_attention(*dp[:7], scale, return_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), plain.view(torch.int16))       # same kernel body, same order of operations
        assert torch.equal(lse, lse_p)
        if whole is not None:
            assert torch.isnan(whole[0]).all() and torch.isnan(whole[-1]).all()   # nothing written outside the problem's rows


def test_group_physical_host_full_size():
    """Physical host 0 of 8 at the 128K configuration: anchor block (2048), virtual host 0 (no passing keys) and
    virtual host 15 (15 passing blocks of 1024), 16384 local tokens each; bit-identical to separate calls, sampled
    rows against the oracle."""
    cfg = wl.CONFIGS["3b-128k"]
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    rng = np.random.default_rng(32)
    scale = 1.0 / math.sqrt(d)
    shapes = [(cfg.l_a, 0, 0), (cfg.L, cfg.l_a, 0), (cfg.L, cfg.l_a, 15 * cfg.l_p)]
    probs = [make_problem(rng, hq, hkv, d, *sh) for sh in shapes]
    dprobs = [tuple(dev(x) for x in pr) for pr in probs]
    res = apbv.apbv_host_attention_group(dprobs, scale)
    torch.cuda.synchronize()
    for m, (pr, dp, out) in enumerate(zip(probs, dprobs, res)):
        plain = apbv.apbv_host_attention(*dp, scale)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), plain.view(torch.int16))
        L = shapes[m][0]
        rows = np.array([0, 255, 256, L // 2 + 3, L - 1])
        ref, _ = oracle.host_attention(*pr, scale, rows=rows)
        check(to_f64(out)[rows], ref, f"physical host, problem {m}, sampled rows")
