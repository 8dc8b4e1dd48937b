"""The library's calls under HIP graph capture: a serving loop records its launch-bound decode
steps (and, for refresh, the eviction pass) once and replays them.  Every replay must give what the
eager call gives, with the program's own eager work and synchronisations between the replays."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
BF16 = synth.BF16


def test_decode_attention_replayed_from_a_graph():
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, S, k, W = 24, 8, 2, 128, 4, 1500, 300
    cap = S + k + W
    key = synth.stream_key(77, 5)
    Kc = synth.host_to_torch(synth.fill_host(key, 0, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d), BF16)
    Vc = synth.host_to_torch(synth.fill_host(key, 1 << 30, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d), BF16)
    q = synth.host_to_torch(synth.fill_host(key, 2 << 30, P * Hq * d, BF16).reshape(P, Hq, d), BF16)
    q2 = synth.host_to_torch(synth.fill_host(key, 3 << 30, P * Hq * d, BF16).reshape(P, Hq, d), BF16)
    desc, ws, out_eager = gu.gpu_decode_setup(BF16, P, Hq, Hkv, d, S, k, W, cap, False)
    out_graph, out_other = torch.zeros_like(out_eager), torch.zeros_like(out_eager)
    sk.sagekv_decode_attn(desc, q, Kc, Vc, cap, out_eager, ws)
    torch.cuda.synchronize()
    want = out_eager.cpu().numpy()
    assert np.isfinite(want).all() and np.abs(want).max() > 0

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sk.sagekv_decode_attn(desc, q, Kc, Vc, cap, out_graph, ws)
    for rep in range(4):
        out_graph.zero_()
        sk.sagekv_decode_attn(desc, q2, Kc, Vc, cap - rep, out_other, ws)  # eager work on the same workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out_graph.cpu().numpy(), want, err_msg=f"replay {rep}")


def test_decode_steps_replayed_from_a_graph():
    """A graph of fused steps (append + attention), replayed from the same starting cache."""
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, S, k, W, steps = 2, 8, 2, 128, 4, 900, 64, 5  # few rows: split rows + combine kernel
    cap = S + k + W
    key = synth.stream_key(78, 5)
    Kc = synth.host_to_torch(synth.fill_host(key, 0, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d), BF16)
    Vc = synth.host_to_torch(synth.fill_host(key, 1 << 30, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d), BF16)
    qs = synth.host_to_torch(synth.fill_host(key, 2 << 30, steps * P * Hq * d, BF16).reshape(steps, P, Hq, d), BF16)
    kn = synth.host_to_torch(synth.fill_host(key, 3 << 30, steps * P * Hkv * d, BF16).reshape(steps, P, Hkv, d), BF16)
    vn = synth.host_to_torch(synth.fill_host(key, 4 << 30, steps * P * Hkv * d, BF16).reshape(steps, P, Hkv, d), BF16)
    desc, ws, _ = gu.gpu_decode_setup(BF16, P, Hq, Hkv, d, S, k, W, cap, False)
    outs_eager = torch.zeros((steps, P, Hq, d), dtype=torch.float32, device="cuda")
    outs_graph = torch.zeros_like(outs_eager)
    Kc_0, Vc_0 = Kc.clone(), Vc.clone()
    Kc_g, Vc_g = Kc.clone(), Vc.clone()
    for t in range(steps):
        sk.sagekv_decode_step(desc, qs[t], kn[t], vn[t], Kc, Vc, t, outs_eager[t], ws)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for t in range(steps):
            sk.sagekv_decode_step(desc, qs[t], kn[t], vn[t], Kc_g, Vc_g, t, outs_graph[t], ws)
    for rep in range(3):
        outs_graph.zero_()
        Kc_g.copy_(Kc_0), Vc_g.copy_(Vc_0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(outs_graph, outs_eager), f"replay {rep}"
        assert torch.equal(Kc_g, Kc) and torch.equal(Vc_g, Vc)


def test_select_replayed_from_a_graph(ref):
    """The eviction pass (pre-filtered path and its gated dense kernels) as one graph."""
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, L, S, W, k = 2, 8, 2, 128, 40000, 4, 128, 1000
    key = synth.stream_key(79, 5)
    q = synth.fill_host(key, 0, P * Hq * d, BF16).reshape(P, Hq, d)
    K = synth.fill_host(key, 1 << 30, P * Hkv * L * d, BF16).reshape(P, Hkv, L, d)
    V = synth.fill_host(key, 1 << 32, P * Hkv * L * d, BF16).reshape(P, Hkv, L, d)
    Kc_r, Vc_r, kept_r = ref.select(BF16, 0, q, K, V, S, W, k)
    qd, Kd, Vd = (synth.host_to_torch(x, BF16) for x in (q, K, V))
    Bt = S + k + W
    desc = sk.select_desc(qd, Kd, Vd, S, W, k, Bt)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=qd.dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.zeros((P, Hkv, Bt), dtype=torch.int32, device="cuda")
    sk.sagekv_select(desc, qd, Kd, Vd, Kc, Vc, kept, None, ws)  # eager once: one-time kernel attributes are set
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kept.cpu().numpy(), kept_r)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sk.sagekv_select(desc, qd, Kd, Vd, Kc, Vc, kept, None, ws)
    for rep in range(3):
        Kc.zero_(), Vc.zero_(), kept.zero_()
        ws.random_(0, 255)  # the pass must not depend on what the workspace held
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(kept.cpu().numpy(), kept_r, err_msg=f"replay {rep}")
        np.testing.assert_array_equal(synth.torch_to_host(Kc, BF16), Kc_r)
        np.testing.assert_array_equal(synth.torch_to_host(Vc, BF16), Vc_r)
        assert sk.sagekv_select_redone_rows(desc, ws) == 0
