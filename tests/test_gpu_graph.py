"""The library's launches under HIP graph capture: a captured (compress + attention) layer step must
replay to the same bits as eager execution, several times, with eager work in between."""
import math

import numpy as np
import pytest
import torch

import paper_2601_21444_amd as apbv
from paper_2601_21444_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def test_layer_step_replays_bit_identically_from_a_hip_graph():
    cfg = wl.custom("graph", 5, 8, 2, 128, 16, 100, 2, 700, 96, 900)
    x = wl.generate(cfg)
    q_probe, q, k_a, v_a, k, v = (dev(a) for a in (x.q_probe, x.q, x.k_anchor, x.v_anchor, x.k, x.v))
    prev = [(dev(a), dev(b)) for a, b in zip(x.k_prev, x.v_prev)]
    scale = 1.0 / math.sqrt(cfg.head_dim)
    hkv, d, lp = cfg.n_kv_heads, cfg.head_dim, cfg.l_p

    ws = torch.empty(apbv.apbv_compress_workspace_bytes(1, hkv, d, cfg.L_prev, lp), dtype=torch.uint8, device="cuda")
    idx = torch.empty((cfg.P, 1, hkv, lp), dtype=torch.int32, device="cuda")
    kp = torch.empty((cfg.P * lp, hkv, d), dtype=torch.bfloat16, device="cuda")
    vp = torch.empty_like(kp)
    out = torch.empty((1, cfg.L, cfg.n_q_heads, d), dtype=torch.bfloat16, device="cuda")

    def step():
        for i, (kb, vb) in enumerate(prev):        # compress the preceding blocks straight into the passing segment
            apbv.apbv_compress_kv(q_probe, kb, vb, lp, workspace=ws, idx_out=idx[i],
                                  k_c_out=kp[i * lp:(i + 1) * lp].unsqueeze(0), v_c_out=vp[i * lp:(i + 1) * lp].unsqueeze(0))
        apbv.apbv_host_attention(q, k_a, v_a, kp, vp, k, v, scale, out=out)

    step()
    torch.cuda.synchronize()
    ref_out, ref_idx, ref_kp = out.clone(), idx.clone(), kp.clone()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                     # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()

    for rep in range(4):
        out.fill_(0)                               # eager work between replays (fill kernels, not memsets in the graph)
        idx.fill_(-1)
        kp.fill_(0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out), f"replay {rep}: attention output differs"
        assert torch.equal(idx, ref_idx) and torch.equal(kp, ref_kp), f"replay {rep}: compression differs"
