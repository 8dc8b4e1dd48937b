"""The decode loop as a serving engine runs it (paper Sec. 2 Step 4, Sec. 4 future work):
the append count lives on the device, so ONE recorded decode step serves every generated token, and
the eviction pass is run again every T tokens into the live reduced cache (interval refresh).
Every call is mirrored in the oracle, step by step."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
BF16, F32 = synth.BF16, synth.F32


def step_inputs(key, t, P, Hq, Hkv, d, dtype):
    q = synth.fill_host(key, (2 << 30) + t * 10_000_000, P * Hq * d, dtype).reshape(P, Hq, d)
    kn = synth.fill_host(key, (3 << 30) + t * 10_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
    vn = synth.fill_host(key, (4 << 30) + t * 10_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
    return q, kn, vn


def random_reduced_cache(key, P, Hkv, cap, d, dtype):
    Kc = synth.fill_host(key, 0, P * Hkv * cap * d, dtype).reshape(P, Hkv, cap, d)
    Vc = synth.fill_host(key, 1 << 30, P * Hkv * cap * d, dtype).reshape(P, Hkv, cap, d)
    return Kc, Vc


@pytest.mark.parametrize(
    "dtype,P,Hq,Hkv,d,S,k,W",
    [
        (BF16, 2, 8, 2, 128, 4, 700, 24),      # few rows: sliced rows, the merge launch moves the count on
        (BF16, 100, 8, 2, 128, 4, 150, 9),     # 200 rows, one workgroup each: the last one to finish does
        (BF16, 150, 14, 2, 128, 3, 100, 7),    # 300 rows, G = 7: 4-wave workgroups
        (BF16, 2, 40, 2, 64, 4, 200, 6),       # G = 20: two launches per step, the second moves the count on
        (BF16, 100, 40, 2, 64, 4, 60, 5),      # the same with one workgroup per row
        (F32, 2, 6, 2, 128, 2, 300, 10),       # fp32 kernel
        (F32, 100, 4, 2, 64, 2, 100, 5),
    ],
)
def test_ring_step_follows_the_oracle_and_the_host_counted_step(ref, dtype, P, Hq, Hkv, d, S, k, W):
    """2 W + 3 steps, across two wraps of the window: every step equals the oracle's (tolerance) and
    the step driven by a host counter (bit for bit); the device count ends every step at t + 1."""
    import torch

    import paper_2503_08879_amd as sk

    Bt = S + k + W
    cap = Bt + 3
    key = synth.stream_key(900 + Hq + P, 66)
    Kc, Vc = random_reduced_cache(key, P, Hkv, cap, d, dtype)
    Kc_d, Vc_d = synth.host_to_torch(Kc, dtype), synth.host_to_torch(Vc, dtype)
    Kc_v, Vc_v = Kc_d.clone(), Vc_d.clone()
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, cap)
    out_v = torch.empty_like(out)
    ring = torch.zeros(2, dtype=torch.int32, device="cuda")
    for t in range(2 * W + 3):
        q, kn, vn = step_inputs(key, t, P, Hq, Hkv, d, dtype)
        ref.append(dtype, Kc, Vc, kn, vn, S + k, W)
        want = ref.decode_attn(dtype, 0, q, Kc, Vc, Bt)
        qd, knd, vnd = (synth.host_to_torch(x, dtype) for x in (q, kn, vn))
        sk.sagekv_decode_step_ring(desc, qd, knd, vnd, Kc_d, Vc_d, ring, out, ws)
        sk.sagekv_decode_step(desc, qd, knd, vnd, Kc_v, Vc_v, t, out_v, ws)
        torch.cuda.synchronize()
        assert ring.tolist() == [t + 1, 0], f"step {t}: ring state {ring.tolist()}"
        err = np.abs(out.cpu().numpy() - want).max()
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: abs err {err:.3e}"
        assert torch.equal(out, out_v), f"step {t}: differs from the host-counted step"
    assert torch.equal(Kc_d, Kc_v) and torch.equal(Vc_d, Vc_v)


@pytest.mark.parametrize("rows_kind", ["sliced", "whole"])
def test_one_recorded_step_serves_every_token(ref, rows_kind):
    """One HIP graph of ONE decode step, replayed 2 W + 3 times (the window wraps twice), with eager
    work of the program between the replays; every replay is compared with the oracle."""
    import torch

    import paper_2503_08879_amd as sk

    dtype = BF16
    P, Hq, Hkv, d, S, k, W = (2, 8, 2, 128, 4, 900, 20) if rows_kind == "sliced" else (100, 8, 2, 128, 4, 120, 11)
    Bt = S + k + W
    cap = Bt
    key = synth.stream_key(950 + P, 66)
    Kc, Vc = random_reduced_cache(key, P, Hkv, cap, d, dtype)
    Kc_d, Vc_d = synth.host_to_torch(Kc, dtype), synth.host_to_torch(Vc, dtype)
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, cap)
    ring = torch.zeros(2, dtype=torch.int32, device="cuda")
    td = synth.torch_dtype(dtype)
    q_buf = torch.zeros((P, Hq, d), dtype=td, device="cuda")
    kn_buf = torch.zeros((P, Hkv, d), dtype=td, device="cuda")
    vn_buf = torch.zeros((P, Hkv, d), dtype=td, device="cuda")
    # unrelated eager work on another cache with the same workspace, between the replays
    Ko, Vo = Kc_d.clone(), Vc_d.clone()
    out_o = torch.empty_like(out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sk.sagekv_decode_step_ring(desc, q_buf, kn_buf, vn_buf, Kc_d, Vc_d, ring, out, ws)
    ring.zero_()
    Kc_d.copy_(synth.host_to_torch(Kc, dtype)), Vc_d.copy_(synth.host_to_torch(Vc, dtype))  # capture ran nothing; be sure
    for t in range(2 * W + 3):
        q, kn, vn = step_inputs(key, t, P, Hq, Hkv, d, dtype)
        ref.append(dtype, Kc, Vc, kn, vn, S + k, W)
        want = ref.decode_attn(dtype, 0, q, Kc, Vc, Bt)
        q_buf.copy_(synth.host_to_torch(q, dtype)), kn_buf.copy_(synth.host_to_torch(kn, dtype))
        vn_buf.copy_(synth.host_to_torch(vn, dtype))
        sk.sagekv_decode_step(desc, q_buf, kn_buf, vn_buf, Ko, Vo, t + 5, out_o, ws)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert ring.tolist() == [t + 1, 0]
        err = np.abs(out.cpu().numpy() - want).max()
        assert err <= gu.DECODE_ATOL[dtype], f"replay {t}: abs err {err:.3e}"
    got_K = synth.torch_to_host(Kc_d, dtype)
    for p in range(P):
        for c in range(Hkv):
            assert sorted(map(bytes, got_K[p, c, S + k:Bt])) == sorted(map(bytes, Kc[p, c, S + k:Bt]))


@pytest.mark.parametrize("P", [2, 100])
def test_ring_step_in_grow_mode(ref, P):
    """Nothing is evicted: rows grow by one token per step until the capacity; then the row stays as it is."""
    import torch

    import paper_2503_08879_amd as sk

    dtype, Hq, Hkv, d, S, k, W, room = BF16, 8, 2, 128, 4, 200, 16, 5
    Bt = S + k + W
    cap = Bt + room
    key = synth.stream_key(970 + P, 66)
    Kc, Vc = random_reduced_cache(key, P, Hkv, cap, d, dtype)
    Kc_d, Vc_d = synth.host_to_torch(Kc, dtype), synth.host_to_torch(Vc, dtype)
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, cap, grow=True)
    ring = torch.zeros(2, dtype=torch.int32, device="cuda")
    length = Bt
    for t in range(room + 2):
        q, kn, vn = step_inputs(key, t, P, Hq, Hkv, d, dtype)
        if length < cap:
            length = ref.append(dtype, Kc, Vc, kn, vn, S + k, W, grow=True, length=length)
        want = ref.decode_attn(dtype, 0, q, Kc, Vc, length)
        sk.sagekv_decode_step_ring(desc, *(synth.host_to_torch(x, dtype) for x in (q, kn, vn)), Kc_d, Vc_d, ring, out, ws)
        torch.cuda.synchronize()
        assert ring.tolist() == [t + 1, 0]
        err = np.abs(out.cpu().numpy() - want).max()
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: abs err {err:.3e}"
    np.testing.assert_array_equal(synth.torch_to_host(Kc_d, dtype), Kc)
    np.testing.assert_array_equal(synth.torch_to_host(Vc_d, dtype), Vc)


@pytest.mark.parametrize("head_mode", [0, 1])
@pytest.mark.parametrize("use_graph", [False, True])
def test_interval_refresh_end_to_end(ref, head_mode, use_graph):
    """Sec. 4, future work: select at L0 -> T decode steps, every generated (k, v) also stored behind
    the prompt in the full cache -> the eviction pass again with the newest token's query over
    L0 + T tokens INTO THE SAME reduced cache and kept_idx -> ring restarted -> T more steps -> a
    second refresh -> more steps.  Kept sets bit-exact and every decode step within tolerance; with
    use_graph the decode steps are replays of one recorded step."""
    import torch

    import paper_2503_08879_amd as sk

    dtype = BF16
    P, Hq, Hkv, d, L0, S, W, k, T = 2, 8, 2, 128, 30000, 4, 48, 600, 70  # T > W: the window wraps before a refresh
    G = Hq // Hkv
    lists = G if head_mode == 1 else 1
    base = S + lists * k
    Bt = base + W
    Lcap = L0 + 2 * T
    key = synth.stream_key(990 + head_mode, 55)
    K = synth.fill_host(key, 1 << 30, P * Hkv * Lcap * d, dtype).reshape(P, Hkv, Lcap, d)
    V = synth.fill_host(key, 1 << 32, P * Hkv * Lcap * d, dtype).reshape(P, Hkv, Lcap, d)
    K[:, :, L0:] = 0  # spare capacity: nothing generated yet
    V[:, :, L0:] = 0
    Kd, Vd = synth.host_to_torch(K, dtype), synth.host_to_torch(V, dtype)
    td = synth.torch_dtype(dtype)
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=td, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    ddesc, dws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, Bt, head_mode=head_mode)
    ring = torch.zeros(2, dtype=torch.int32, device="cuda")
    q_buf = torch.zeros((P, Hq, d), dtype=td, device="cuda")
    kn_buf = torch.zeros((P, Hkv, d), dtype=td, device="cuda")
    vn_buf = torch.zeros((P, Hkv, d), dtype=td, device="cuda")
    graph = None
    if use_graph:
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            sk.sagekv_decode_step_ring(ddesc, q_buf, kn_buf, vn_buf, Kc, Vc, ring, out, dws)
        ring.zero_(), Kc.zero_(), Vc.zero_()

    def evict(L, q_now):
        """The eviction pass over the first L tokens on both sides; returns the oracle's reduced cache."""
        sdesc = sk.select_desc(synth.host_to_torch(q_now, dtype), Kd[:, :, :L], Vd[:, :, :L], S, W, k, Bt,
                               head_mode=head_mode)
        ws = torch.empty(sk.sagekv_select_workspace_bytes(sdesc), dtype=torch.uint8, device="cuda")
        sk.sagekv_select(sdesc, synth.host_to_torch(q_now, dtype), Kd[:, :, :L], Vd[:, :, :L], Kc, Vc, kept, None, ws)
        ring.zero_()  # the caller's part of a refresh: the window is in position order again
        torch.cuda.synchronize()
        Kc_r, Vc_r, kept_r, s_r = ref.select(dtype, head_mode, q_now, np.ascontiguousarray(K[:, :, :L]),
                                             np.ascontiguousarray(V[:, :, :L]), S, W, k, want_scores=True)
        got = kept.cpu().numpy()
        for li in range(lists):
            cut = lambda a: np.concatenate([a[..., :S], a[..., S + li * k:S + (li + 1) * k], a[..., base:]], axis=-1)
            assert gu.check_kept(cut(got), cut(kept_r), s_r[:, :, li], S, W, k) == 0
        np.testing.assert_array_equal(synth.torch_to_host(Kc, dtype), Kc_r)
        np.testing.assert_array_equal(synth.torch_to_host(Vc, dtype), Vc_r)
        return Kc_r, Vc_r, kept_r

    q_now = synth.fill_host(key, 0, P * Hq * d, dtype).reshape(P, Hq, d)
    L = L0
    Kc_r, Vc_r, kept_prev = evict(L, q_now)
    step = 0
    for phase, n_steps in enumerate((T, T, 5)):
        for i in range(n_steps):
            q, kn, vn = step_inputs(key, step, P, Hq, Hkv, d, dtype)
            step += 1
            ref.append(dtype, Kc_r, Vc_r, kn, vn, base, W)
            want = ref.decode_attn(dtype, head_mode, q, Kc_r, Vc_r, Bt, S, k, W)
            q_buf.copy_(synth.host_to_torch(q, dtype)), kn_buf.copy_(synth.host_to_torch(kn, dtype))
            vn_buf.copy_(synth.host_to_torch(vn, dtype))
            if L < Lcap:  # the caller keeps the full cache up to date: the generated token joins it
                K[:, :, L], V[:, :, L] = kn, vn
                Kd[:, :, L].copy_(kn_buf), Vd[:, :, L].copy_(vn_buf)
                L += 1
            if graph is not None:
                torch.cuda.synchronize()
                graph.replay()
            else:
                sk.sagekv_decode_step_ring(ddesc, q_buf, kn_buf, vn_buf, Kc, Vc, ring, out, dws)
            torch.cuda.synchronize()
            assert ring.tolist() == [i + 1, 0]
            err = np.abs(out.cpu().numpy() - want).max()
            assert err <= gu.DECODE_ATOL[dtype], f"phase {phase} step {i}: abs err {err:.3e}"
            q_now = q
        if phase < 2:
            assert L == L0 + (phase + 1) * T
            Kc_r, Vc_r, kept_now = evict(L, q_now)  # refresh with the newest token's query
            assert not np.array_equal(kept_now, kept_prev)
            # the T generated tokens are the newest of the cache: all inside the new recent window or candidates
            assert kept_now[0, 0, -1] == L - 1
            kept_prev = kept_now
