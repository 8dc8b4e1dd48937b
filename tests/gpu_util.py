"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding on host arrays,
and compare with the oracle to the stated bar."""
from __future__ import annotations

import numpy as np

import synth

SCORE_RTOL = 1e-5          # fp32 scores vs oracle, relative
TIE_RTOL = 1e-6            # kept-set exemption band around the oracle's k-th score
DECODE_ATOL = {synth.BF16: 2e-2, synth.F32: 1e-5}


def have_gpu() -> bool:
    import torch

    return torch.cuda.is_available()


def gpu_select(dtype, q, K, V, S, W, k, cap=None, want_scores=True, K_dev=None, V_dev=None, flags=0, head_mode=0):
    """q [P,Hq,d], K/V [P,Hkv,L,d] host arrays (or device tensors via K_dev/V_dev).
    Returns dict of host arrays: Kc, Vc, kept, scores."""
    import torch

    import paper_2503_08879_amd as sk

    qd = synth.host_to_torch(q, dtype)
    Kd = K_dev if K_dev is not None else synth.host_to_torch(K, dtype)
    Vd = V_dev if V_dev is not None else synth.host_to_torch(V, dtype)
    P, Hq, d = qd.shape
    Hkv, L = Kd.shape[1], Kd.shape[2]
    lists = Hq // Hkv if head_mode == 1 else 1
    n_kept = S + lists * k + W
    cap = n_kept if cap is None else cap
    desc = sk.select_desc(qd, Kd, Vd, S, W, k, cap, flags=flags, head_mode=head_mode)
    ws = torch.empty(max(sk.sagekv_select_workspace_bytes(desc), 16), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, cap, d), dtype=Kd.dtype, device="cuda")
    Vc = torch.zeros((P, Hkv, cap, d), dtype=Kd.dtype, device="cuda")
    kept = torch.full((P, Hkv, n_kept), -1, dtype=torch.int32, device="cuda")
    scores = torch.empty((P, Hkv * lists, L), dtype=torch.float32, device="cuda") if want_scores else None
    sk.sagekv_select(desc, qd, Kd, Vd, Kc, Vc, kept, scores, ws)
    torch.cuda.synchronize()
    return {
        "redone": sk.sagekv_select_redone_rows(desc, ws),
        "Kc": synth.torch_to_host(Kc, dtype), "Vc": synth.torch_to_host(Vc, dtype), "kept": kept.cpu().numpy(),
        "scores": None if scores is None else scores.cpu().numpy(), "Kc_dev": Kc, "Vc_dev": Vc,
    }


def check_scores(got, want, cand=None):
    """got, want: fp32 [..., L]."""
    g, w = got.astype(np.float64), want.astype(np.float64)
    rel = np.abs(g - w) / np.maximum(np.abs(w), 1e-300)
    assert rel.max() <= SCORE_RTOL, f"score rel err {rel.max():.3e}"


def check_kept(kept_gpu, kept_ref, scores_ref, S, W, k):
    """Bit-exact kept sets, except that a token may be swapped for another one when both have an
    oracle score within TIE_RTOL (relative) of the oracle's k-th score.  Returns #rows that used the exemption."""
    kept_gpu = kept_gpu.reshape(-1, kept_gpu.shape[-1])
    kept_ref = kept_ref.reshape(-1, kept_ref.shape[-1])
    s = scores_ref.reshape(kept_ref.shape[0], -1)
    exempt_rows = 0
    for r in range(kept_ref.shape[0]):
        a, b = kept_gpu[r], kept_ref[r]
        assert np.array_equal(a[:S], b[:S]) and np.array_equal(a[S + k:], b[S + k:]), f"row {r}: sink/recent differ"
        if np.array_equal(a, b):
            continue
        sa, sb = a[S:S + k], b[S:S + k]
        assert np.all(np.diff(sa) > 0), f"row {r}: selected indices not ascending"
        L = s.shape[1]
        assert sa.min() >= S and sa.max() < L - W
        only_gpu, only_ref = np.setdiff1d(sa, sb), np.setdiff1d(sb, sa)
        assert len(only_gpu) == len(only_ref)
        kth = float(np.sort(s[r, S:L - W].astype(np.float64))[::-1][k - 1])
        for i in np.concatenate([only_gpu, only_ref]):
            rel = abs(float(s[r, i]) - kth) / kth
            assert rel <= TIE_RTOL, f"row {r}: token {i} differs, score {s[r, i]!r} vs k-th {kth!r} (rel {rel:.2e})"
        exempt_rows += 1
    return exempt_rows


def check_gather(out, K, V, S, k, W):
    """Kc/Vc rows equal K/V at the GPU's own kept indices, byte for byte."""
    kept = out["kept"]
    P, Hkv, n = kept.shape
    for p in range(P):
        for c in range(Hkv):
            np.testing.assert_array_equal(out["Kc"][p, c, :n], K[p, c][kept[p, c]])
            np.testing.assert_array_equal(out["Vc"][p, c, :n], V[p, c][kept[p, c]])


def gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, cap, grow=False, head_mode=0):
    import torch

    import paper_2503_08879_amd as sk

    desc = sk.decode_desc(P, Hq, Hkv, d, dtype, S, k, W, cap, grow, head_mode=head_mode)
    ws = torch.empty(max(sk.sagekv_decode_workspace_bytes(desc), 16), dtype=torch.uint8, device="cuda")
    out = torch.empty((P, Hq, d), dtype=torch.float32, device="cuda")
    return desc, ws, out
