"""GPU parity at the documented size limits of the ABI: a context block of 2^24 tokens (the largest token count a view
may have) through the compression, and key/value views whose token stride is the largest allowed (just below 2^24
elements, so that the kernels' 32-bit row offsets inside a tile are at their bound) through the attention."""
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
    return wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def test_compress_block_of_2_pow_24_tokens():
    """L = 2^24, one KV head, d = 64: indices bit-exact against the oracle.  The block is 64 copies of a 2^18-token
    random block, so every score occurs 64 times: the selection is decided by the tie rule at every rank."""
    rng = np.random.default_rng(81)
    L, d, n_q, l_p = 1 << 24, 64, 3, 1000
    base = rand_bits(rng, (1 << 18, 1, d))
    k = np.tile(base, (64, 1, 1))
    qp = rand_bits(rng, (n_q, 2, d))
    print("compress limit case: L = 2^24", flush=True)
    dk = dev(k)
    idx, k_c, v_c, s = apbv.apbv_compress_kv(dev(qp), dk, dk, l_p, return_scores=True)
    torch.cuda.synchronize()
    s_ref = oracle.importance_scores(qp, k)
    np.testing.assert_allclose(s.cpu().numpy(), s_ref, rtol=1e-12, atol=1e-12)
    want = oracle.arg_top(s_ref[0], l_p)
    np.testing.assert_array_equal(idx.cpu().numpy()[0], want)
    got_rows = k_c.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)[:, 0]
    np.testing.assert_array_equal(got_rows, k[want, 0])


def test_attention_with_the_largest_token_stride():
    """Passing keys and values viewed with stride_token = 2^24 - 8 elements (32 MB between consecutive tokens)."""
    rng = np.random.default_rng(82)
    hq, hkv, d, L, l_a, n_p = 2, 1, 128, 70, 5, 130
    st = (1 << 24) - 8
    scale = 1.0 / math.sqrt(d)
    q = rand_bits(rng, (L, hq, d))
    ka, va, kp, vp, k, v = (rand_bits(rng, (n, hkv, d)) for n in (l_a, l_a, n_p, n_p, L, L))
    print("attention limit case: stride_token = 2^24 - 8", flush=True)
    big_k = torch.zeros((n_p - 1) * st + hkv * d, dtype=torch.bfloat16, device="cuda")
    big_v = torch.zeros_like(big_k)
    kp_view = torch.as_strided(big_k, (n_p, hkv, d), (st, d, 1))
    vp_view = torch.as_strided(big_v, (n_p, hkv, d), (st, d, 1))
    kp_view.copy_(dev(kp))
    vp_view.copy_(dev(vp))
    out, lse = apbv.apbv_host_attention(dev(q), dev(ka), dev(va), kp_view, vp_view, dev(k), dev(v), scale, return_lse=True)
    torch.cuda.synchronize()
    ref, lse_r = oracle.host_attention(q, ka, va, kp, vp, k, v, scale)
    diff = np.abs(to_f64(out) - ref)
    assert diff.max() <= 2e-2 and diff.mean() / np.abs(ref).mean() <= 5e-3
    np.testing.assert_allclose(lse.cpu().numpy().astype(np.float64), lse_r, atol=2e-3, rtol=0)
    # one element more is refused before anything is launched
    too_wide = torch.as_strided(big_k, (2, hkv, d), (1 << 24, d, 1))
    with pytest.raises(apbv.ApbvError):
        apbv.apbv_host_attention(dev(q), dev(ka), dev(va), too_wide, too_wide, dev(k), dev(v), scale)
