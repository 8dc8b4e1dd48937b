"""Full-size configurations, in the launch configuration bench.py times (all layers in one call,
no scores_out, fused decode steps).  The host cannot hold these caches at once, so the oracle works
through them one problem (layer x sequence) at a time, on K and V copied back from the device (the
device fill is bit-identical to the host fill: test_device_fill_equals_host_fill,
test_device_config_equals_host_config): EVERY row's kept set and gathered K/V is compared with the
oracle's, and the decode steps run against the oracle's own reduced cache."""
import time

import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
GROUP_SUM = 0


def host_problem(cfg, p, pos, nrows):
    """K, V of problem p regenerated on the host: [1, Hkv, L, d] each."""
    rows = range(p * cfg.n_kv_heads, (p + 1) * cfg.n_kv_heads)
    K = np.stack([synth.kv_row_host(cfg, "K", r, pos, nrows) for r in rows])[None]
    V = np.stack([synth.kv_row_host(cfg, "V", r) for r in rows])[None]
    return K, V


def full_size_case(ref, cfg, problems, n_decode):
    import torch

    import paper_2503_08879_amd as sk

    S, W, k, Bt = cfg.n_sink, cfg.n_recent, cfg.k, cfg.budget
    P, Hq, Hkv, d, L = cfg.n_problems, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.L
    q_last, K, V, pos = synth.kv_device(cfg)
    td = synth.torch_dtype(cfg.dtype)
    desc = sk.select_desc(q_last, K, V, S, W, k, Bt)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=td, device="cuda")
    Vc = torch.zeros((P, Hkv, Bt, d), dtype=td, device="cuda")
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    sk.sagekv_select(desc, q_last, K, V, Kc, Vc, kept, None, ws)
    torch.cuda.synchronize()
    redone = sk.sagekv_select_redone_rows(desc, ws)
    print(f"{cfg.name}: rows redone by the dense path: {redone} of {cfg.rows}", flush=True)

    # ---- every row: structure of the kept set, all needles kept, gather is a byte copy
    kept_h = kept.cpu().numpy().reshape(cfg.rows, Bt)
    assert np.array_equal(kept_h[:, :S], np.tile(np.arange(S), (cfg.rows, 1)))
    assert np.array_equal(kept_h[:, S + k:], np.tile(np.arange(L - W, L), (cfg.rows, 1)))
    sel = kept_h[:, S:S + k]
    assert np.all(np.diff(sel, axis=1) > 0) and sel.min() >= S and sel.max() < L - W
    # where a needle (logit ~ 3 on one head) is far above the k-th score, recall must be 100 %;
    # in the other configs (k/E around 1 %, G = 7, or scale U[2,4]) some needles sit near the threshold
    if cfg.name == "C2":
        for r in range(cfg.rows):
            assert np.isin(pos[r], sel[r]).all(), f"row {r} lost a needle"
    idx = kept.to(torch.int64).view(cfg.rows, Bt, 1).expand(-1, -1, d)
    assert torch.equal(torch.gather(K.view(cfg.rows, L, d), 1, idx), Kc.view(cfg.rows, Bt, d))
    assert torch.equal(torch.gather(V.view(cfg.rows, L, d), 1, idx), Vc.view(cfg.rows, Bt, d))
    del idx

    # ---- the oracle's kept set and reduced cache, problem by problem, on the device's own K and V
    qh = synth.q_last_host(cfg)
    Kc_h, Vc_h = synth.torch_to_host(Kc, cfg.dtype), synth.torch_to_host(Vc, cfg.dtype)
    refs = {}
    n_exempt, t0 = 0, time.time()
    for i, p in enumerate(problems):
        Kp, Vp = synth.torch_to_host(K[p:p + 1], cfg.dtype), synth.torch_to_host(V[p:p + 1], cfg.dtype)
        Kc_r, Vc_r, kept_r, s_r = ref.select(cfg.dtype, GROUP_SUM, qh[p:p + 1], Kp, Vp, S, W, k, want_scores=True)
        n_ex = gu.check_kept(kept_h[p * Hkv:(p + 1) * Hkv], kept_r, s_r[:, :, 0], S, W, k)
        n_exempt += n_ex
        if n_ex == 0:
            np.testing.assert_array_equal(Kc_h[p:p + 1], Kc_r)
            np.testing.assert_array_equal(Vc_h[p:p + 1], Vc_r)
            refs[p] = (Kc_r, Vc_r)
        del Kp, Vp
        if i % 16 == 15:
            print(f"{cfg.name}: {i + 1} of {len(problems)} problems equal the oracle's ({time.time() - t0:.0f} s)", flush=True)
    print(f"{cfg.name}: kept sets of {len(problems) * Hkv} rows compared with the oracle, {n_exempt} rows used the "
          f"1e-6 near-tie exemption", flush=True)
    assert n_exempt <= max(1, len(problems) * Hkv // 50)
    del K, V, Kc_h, Vc_h

    # ---- decode steps: every compared problem against the oracle's own reduced cache
    ddesc = sk.decode_desc(P, Hq, Hkv, d, cfg.dtype, S, k, W, Bt)
    dws = torch.empty(max(sk.sagekv_decode_workspace_bytes(ddesc), 16), dtype=torch.uint8, device="cuda")
    out = torch.empty((P, Hq, d), dtype=torch.float32, device="cuda")
    worst = 0.0
    for t in range(n_decode):
        qs, kn, vn = synth.decode_inputs_host(cfg, t)
        qd, knd, vnd = (synth.host_to_torch(x, cfg.dtype) for x in (qs, kn, vn))
        sk.sagekv_decode_step(ddesc, qd, knd, vnd, Kc, Vc, t, out, dws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        for p, (Kc_r, Vc_r) in refs.items():
            ref.append(cfg.dtype, Kc_r, Vc_r, kn[p:p + 1], vn[p:p + 1], S + k, W)
            want = ref.decode_attn(cfg.dtype, GROUP_SUM, qs[p:p + 1], Kc_r, Vc_r, Bt)
            err = np.abs(got[p:p + 1] - want).max()
            worst = max(worst, float(err))
            assert err <= gu.DECODE_ATOL[cfg.dtype], f"problem {p} step {t}: {err:.3e}"
        if t % 32 == 31:
            print(f"{cfg.name}: {t + 1} decode steps, worst abs error so far {worst:.2e}", flush=True)
    # after more steps than the window holds, every original recent token has left: the rings hold the same rows
    if n_decode:
        got_K = synth.torch_to_host(Kc, cfg.dtype)
        for p, (Kc_r, _) in refs.items():
            for c in range(Hkv):
                assert sorted(map(bytes, got_K[p, c, S + k:Bt])) == sorted(map(bytes, Kc_r[0, c, S + k:Bt]))
    print(f"{cfg.name}: {n_decode} decode steps on {len(refs)} problems, worst abs error {worst:.2e}", flush=True)
    return redone


def test_C2_full(ref):
    """Every row against the oracle; decode through more than one full turn of the recent ring (W = 256)."""
    cfg = synth.CONFIGS["C2"]
    assert full_size_case(ref, cfg, problems=range(cfg.n_problems), n_decode=cfg.n_recent + 4) == 0


def test_C3_full(ref):
    cfg = synth.CONFIGS["C3"]
    assert full_size_case(ref, cfg, problems=range(cfg.n_problems), n_decode=6) == 0


def test_C4_full(ref):
    """Qwen2.5-7B shape: G = 7, 28 layers x 4 sequences = 112 problems of L = 131072; W = 128, so the
    decode steps take the ring through a full turn here too."""
    cfg = synth.CONFIGS["C4"]
    assert full_size_case(ref, cfg, problems=range(cfg.n_problems), n_decode=cfg.n_recent + 2) == 0


def test_C5_full(ref):
    """ProLong shape: L = 524288, 32 layers resident (64 GiB of K and V); every row against the oracle."""
    cfg = synth.CONFIGS["C5"]
    # needles at log-uniform positions crowd the first tokens of every row; a row whose sample is
    # dominated by them cannot be certified and is redone densely (same result, checked above)
    assert full_size_case(ref, cfg, problems=range(cfg.n_problems), n_decode=4) <= cfg.rows // 10


def test_C4_per_query_paper_budget_full(ref):
    """The appendix's own setting for Qwen2.5-7B (App. A.2): B = 8192 -> sink 2048, 512 per query head
    (7 lists per KV head), recent 2560, one top-k per query head, on the full C4 cache."""
    import torch

    import paper_2503_08879_amd as sk

    base = synth.CONFIGS["C4"]
    S, k, W = ref.paper_budget(8192, base.G)
    assert (S, k, W) == (2048, 512, 2560)
    cfg = base.with_(n_sink=S, k=k, n_recent=W)
    G, P, Hq, Hkv, d, L = cfg.G, cfg.n_problems, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.L
    Bt = S + G * k + W
    q_last, K, V, pos = synth.kv_device(cfg)
    desc = sk.select_desc(q_last, K, V, S, W, k, Bt, head_mode=sk.PER_QUERY)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=K.dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    sk.sagekv_select(desc, q_last, K, V, Kc, Vc, kept, None, ws)
    torch.cuda.synchronize()
    redone = sk.sagekv_select_redone_rows(desc, ws)
    print(f"C4 per-query B=8192: rows redone by the dense path: {redone} of {cfg.rows}", flush=True)
    assert redone == 0
    kept_h = kept.cpu().numpy().reshape(cfg.rows, Bt)
    assert np.array_equal(kept_h[:, :S], np.tile(np.arange(S), (cfg.rows, 1)))
    assert np.array_equal(kept_h[:, S + G * k:], np.tile(np.arange(L - W, L), (cfg.rows, 1)))
    for g in range(G):
        sel = kept_h[:, S + g * k:S + (g + 1) * k]
        assert np.all(np.diff(sel, axis=1) > 0) and sel.min() >= S and sel.max() < L - W
    idx = kept.to(torch.int64).view(cfg.rows, Bt, 1).expand(-1, -1, d)
    assert torch.equal(torch.gather(K.view(cfg.rows, L, d), 1, idx), Kc.view(cfg.rows, Bt, d))
    assert torch.equal(torch.gather(V.view(cfg.rows, L, d), 1, idx), Vc.view(cfg.rows, Bt, d))
    del idx
    qh = synth.q_last_host(cfg)
    refs = {}
    Kc_h, Vc_h = synth.torch_to_host(Kc, cfg.dtype), synth.torch_to_host(Vc, cfg.dtype)
    for p in range(0, P, 7):  # 16 of the 112 problems, every sequence of the batch among them
        Kp, Vp = synth.torch_to_host(K[p:p + 1], cfg.dtype), synth.torch_to_host(V[p:p + 1], cfg.dtype)
        Kc_r, Vc_r, kept_r, s_r = ref.select(cfg.dtype, 1, qh[p:p + 1], Kp, Vp, S, W, k, want_scores=True)
        got = kept_h[p * Hkv:(p + 1) * Hkv]
        n_ex = 0
        for g in range(G):
            cut = lambda a: np.concatenate([a[..., :S], a[..., S + g * k:S + (g + 1) * k], a[..., S + G * k:]], axis=-1)
            n_ex += gu.check_kept(cut(got), cut(kept_r.reshape(Hkv, Bt)), s_r[0][:, g], S, W, k)
        if n_ex == 0:
            np.testing.assert_array_equal(Kc_h[p:p + 1], Kc_r)
            np.testing.assert_array_equal(Vc_h[p:p + 1], Vc_r)
            refs[p] = (Kc_r, Vc_r)
    assert len(refs) >= 12
    del K, V, Kc_h, Vc_h
    # decode: head g attends the sink, its own list and the recent window
    ddesc = sk.decode_desc(P, Hq, Hkv, d, cfg.dtype, S, k, W, Bt, head_mode=sk.PER_QUERY)
    dws = torch.empty(max(sk.sagekv_decode_workspace_bytes(ddesc), 16), dtype=torch.uint8, device="cuda")
    out = torch.empty((P, Hq, d), dtype=torch.float32, device="cuda")
    for t in range(4):
        qs, kn, vn = synth.decode_inputs_host(cfg, t)
        sk.sagekv_decode_step(ddesc, *(synth.host_to_torch(x, cfg.dtype) for x in (qs, kn, vn)), Kc, Vc, t, out, dws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for p, (Kc_r, Vc_r) in refs.items():
            ref.append(cfg.dtype, Kc_r, Vc_r, kn[p:p + 1], vn[p:p + 1], S + G * k, W)
            want = ref.decode_attn(cfg.dtype, 1, qs[p:p + 1], Kc_r, Vc_r, 0, S, k, W)
            err = np.abs(got[p:p + 1] - want).max()
            assert err <= gu.DECODE_ATOL[cfg.dtype], f"problem {p} step {t}: {err:.3e}"


def test_C5_length_dense_path(ref):
    """The dense path (every token's score written, multi-workgroup histograms, bitmap top-k) at the
    longest configured row, L = 524288, on two layers; kept sets and scores against the oracle."""
    import torch

    import paper_2503_08879_amd as sk

    cfg = synth.CONFIGS["C5"].with_(n_layers=2)
    S, W, k, Bt = cfg.n_sink, cfg.n_recent, cfg.k, cfg.budget
    P, Hkv, d, L = cfg.n_problems, cfg.n_kv_heads, cfg.head_dim, cfg.L
    q_last, K, V, pos = synth.kv_device(cfg)
    desc = sk.select_desc(q_last, K, V, S, W, k, Bt)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=K.dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    scores = torch.empty((P, Hkv, L), dtype=torch.float32, device="cuda")
    sk.sagekv_select(desc, q_last, K, V, Kc, Vc, kept, scores, ws)
    torch.cuda.synchronize()
    assert sk.sagekv_select_redone_rows(desc, ws) == -1
    qh = synth.q_last_host(cfg)
    _, nrows = synth.needles(cfg, qh)
    p = 1
    Kp, Vp = host_problem(cfg, p, pos, nrows)  # regenerated on the host: the device fill at full row length
    np.testing.assert_array_equal(synth.torch_to_host(K[p:p + 1], cfg.dtype), Kp)
    Kc_r, Vc_r, kept_r, s_r = ref.select(cfg.dtype, GROUP_SUM, qh[p:p + 1], Kp, Vp, S, W, k, want_scores=True)
    gu.check_scores(scores[p:p + 1].cpu().numpy(), s_r[:, :, 0])
    n_ex = gu.check_kept(kept[p].cpu().numpy(), kept_r, s_r[:, :, 0], S, W, k)
    if n_ex == 0:
        np.testing.assert_array_equal(synth.torch_to_host(Kc[p:p + 1], cfg.dtype), Kc_r)
        np.testing.assert_array_equal(synth.torch_to_host(Vc[p:p + 1], cfg.dtype), Vc_r)
    # the pre-filtered pass over the same cache keeps the same tokens
    sk.sagekv_select(desc, q_last, K, V, Kc, Vc, torch.zeros_like(kept), None, ws)
    kept2 = torch.zeros_like(kept)
    sk.sagekv_select(desc, q_last, K, V, Kc, Vc, kept2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(kept2, kept)


@pytest.mark.parametrize("scale", [5.0, 12.0, 40.0])
def test_peaked_attention_at_full_length(ref, scale):
    """Queries scaled until a handful of tokens hold the whole softmax (logits of magnitude up to
    ~150): each head's normaliser is then a sum of very few fp32-rounded terms, the case where its error
    is largest.  64 rows of L = 131072 in the C3 split, every kept set and the gathered K/V against the oracle."""
    P, Hq, Hkv, d, L, S, W, k = 8, 32, 8, 128, 131072, 4, 512, 3580
    key = synth.stream_key(4242, 55)
    q = synth.fill_host(key, 0, P * Hq * d, 0).reshape(P, Hq, d)
    q = synth.round_to_dtype(scale * synth.to_f64(q, 0), 0)
    K = synth.fill_host(key, 1 << 30, P * Hkv * L * d, 0).reshape(P, Hkv, L, d)
    V = synth.fill_host(key, 1 << 33, P * Hkv * L * d, 0).reshape(P, Hkv, L, d)
    Kc_r, Vc_r, kept_r, s_r = ref.select(0, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    out = gu.gpu_select(0, q, K, V, S, W, k, want_scores=False)
    print(f"scale {scale}: rows redone by the dense path: {out['redone']} of {P * Hkv}", flush=True)
    if gu.check_kept(out["kept"], kept_r, s_r[:, :, 0], S, W, k) == 0:
        np.testing.assert_array_equal(out["Kc"], Kc_r)
        np.testing.assert_array_equal(out["Vc"], Vc_r)
