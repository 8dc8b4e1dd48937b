"""Pins of the CPU oracle against what the paper and the mathematics fix.

Every check here compares the oracle with something other than itself: a brute-force
sort, a closed form, an invariant the paper states, or a library routine on a special
case.  No GPU, no HIP code.
"""
import math
import os

import numpy as np
import pytest
import torch

import synth

BF16, F32 = 0, 1
GROUP_SUM, PER_QUERY = 0, 1


def rand_inputs(seed, P, Hq, Hkv, d, L, dtype):
    key = synth.stream_key(seed, 77)
    q = synth.fill_host(key, 0, P * Hq * d, dtype).reshape(P, Hq, d)
    K = synth.fill_host(key, 10_000_000, P * Hkv * L * d, dtype).reshape(P, Hkv, L, d)
    V = synth.fill_host(key, 90_000_000, P * Hkv * L * d, dtype).reshape(P, Hkv, L, d)
    return q, K, V


def np_probs(q, K, dtype):
    """Library fp64 softmax(q K^T / sqrt(d)) with consecutive GQA grouping: [P,Hq,L]."""
    q64 = torch.from_numpy(synth.to_f64(q, dtype))
    K64 = torch.from_numpy(synth.to_f64(K, dtype))
    P, Hq, d = q64.shape
    Hkv = K64.shape[1]
    G = Hq // Hkv
    Kh = K64.repeat_interleave(G, dim=1)  # head h reads KV head h // G
    logits = torch.einsum("phd,phld->phl", q64, Kh) / math.sqrt(d)
    return torch.softmax(logits, dim=-1).numpy()


def brute_topk(s32, S, W, k):
    """Full sort of (-score, index) over the candidates; first k, ascending."""
    L = len(s32)
    cands = sorted(range(S, L - W), key=lambda i: (-float(s32[i]), i))
    return sorted(cands[:k])


# ------------------------------------------------------------------ scores
@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (7, 1), (3, 3)])
def test_scores_equal_library_softmax(ref, dtype, Hq, Hkv):
    q, K, _ = rand_inputs(1, 2, Hq, Hkv, 16, 50, dtype)
    p = np_probs(q, K, dtype)  # [P,Hq,L]
    G = Hq // Hkv
    s_pq = ref.scores(dtype, PER_QUERY, q, K)  # [P,Hkv,G,L]
    np.testing.assert_array_equal(s_pq.reshape(2, Hq, 50), p.astype(np.float32))
    s_gs = ref.scores(dtype, GROUP_SUM, q, K)[:, :, 0]  # [P,Hkv,L]
    want = p.reshape(2, Hkv, G, 50)
    acc = np.zeros((2, Hkv, 50))
    for g in range(G):  # ascending g, one rounding at the end
        acc = acc + want[:, :, g]
    np.testing.assert_allclose(s_gs, acc.astype(np.float32), rtol=2e-7, atol=0)


def test_softmax_rows_sum_to_one(ref):
    q, K, _ = rand_inputs(2, 1, 8, 2, 32, 1000, F32)
    s = ref.scores(F32, PER_QUERY, q, K).astype(np.float64)
    np.testing.assert_allclose(s.sum(-1), 1.0, rtol=0, atol=1e-6)  # fp32-rounded terms
    sg = ref.scores(F32, GROUP_SUM, q, K).astype(np.float64)
    np.testing.assert_allclose(sg.sum(-1), 4.0, rtol=0, atol=4e-6)


def test_one_hot_closed_form(ref):
    """q = a e_0, K[i] = b_i e_0  =>  p_i = exp(a b_i / sqrt(d)) / sum_j exp(a b_j / sqrt(d))."""
    d, L, a = 16, 33, 1.75
    b = np.linspace(-2.0, 3.0, L)
    q = np.zeros((1, 1, d), np.float32)
    q[0, 0, 0] = a
    K = np.zeros((1, 1, L, d), np.float32)
    K[0, 0, :, 0] = b.astype(np.float32)
    e = np.exp(a * b.astype(np.float32).astype(np.float64) / math.sqrt(d))
    want = (e / e.sum()).astype(np.float32)
    got = ref.scores(F32, PER_QUERY, q, K)[0, 0, 0]
    np.testing.assert_allclose(got, want, rtol=3e-7)
    # a dropped 1/sqrt(d) or a transposed K would change the ratio p_max/p_min
    assert abs(math.log(got[-1] / got[0]) - a * 5.0 / math.sqrt(d)) < 1e-5


def test_shift_invariance(ref):
    """Adding c*q to every key adds a constant to every logit: probabilities unchanged."""
    q, K, _ = rand_inputs(3, 1, 1, 1, 8, 40, F32)
    K2 = (K + 0.5 * q[:, :, None, :]).astype(np.float32)
    a = ref.scores(F32, PER_QUERY, q, K)
    b = ref.scores(F32, PER_QUERY, q, K2)
    np.testing.assert_allclose(a, b, rtol=2e-5)


# ------------------------------------------------------------------ top-k / partition
@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("mode", [GROUP_SUM, PER_QUERY])
def test_brute_force_topk_all_k(ref, dtype, mode):
    P, Hq, Hkv, d, L, S, W = 2, 4, 2, 8, 40, 3, 5
    q, K, V = rand_inputs(4, P, Hq, Hkv, d, L, dtype)
    G = Hq // Hkv
    E = L - S - W
    p = np_probs(q, K, dtype).reshape(P, Hkv, G, L)
    for k in range(0, E + 1):
        Kc, Vc, kept = ref.select(dtype, mode, q, K, V, S, W, k)
        for pi in range(P):
            for c in range(Hkv):
                if mode == GROUP_SUM:
                    acc = np.zeros(L)
                    for g in range(G):
                        acc = acc + p[pi, c, g]
                    lists = [brute_topk(acc.astype(np.float32), S, W, k)]
                else:
                    lists = [brute_topk(p[pi, c, g].astype(np.float32), S, W, k) for g in range(G)]
                want = list(range(S)) + [i for l in lists for i in l] + list(range(L - W, L))
                assert kept[pi, c].tolist() == want, (k, pi, c)
                np.testing.assert_array_equal(Kc[pi, c], K[pi, c][want])
                np.testing.assert_array_equal(Vc[pi, c], V[pi, c][want])


def test_zero_query_ties_go_to_lower_index(ref):
    q, K, V = rand_inputs(5, 1, 4, 2, 8, 64, F32)
    q[:] = 0
    S, W, k = 4, 8, 11
    _, _, kept = ref.select(F32, GROUP_SUM, q, K, V, S, W, k)
    want = list(range(S + k)) + list(range(64 - W, 64))
    assert kept[0, 0].tolist() == want and kept[0, 1].tolist() == want


def test_duplicate_key_across_boundary_keeps_lower_index(ref):
    """Two identical K rows have identical scores; with exactly one slot left the lower index wins."""
    L, S, W, d = 32, 2, 4, 8
    q, K, V = rand_inputs(6, 1, 1, 1, d, L, F32)
    s = ref.scores(F32, PER_QUERY, q, K)[0, 0, 0]
    order = sorted(range(S, L - W), key=lambda i: (-float(s[i]), i))
    k = 5
    a = order[k - 1]  # the k-th best candidate
    b = 20 if a != 20 else 21  # copy it to another candidate position
    K[0, 0, b] = K[0, 0, a]
    _, _, kept = ref.select(F32, PER_QUERY, q, K, V, S, W, k)
    sel = set(kept[0, 0, S:S + k].tolist())
    s2 = ref.scores(F32, PER_QUERY, q, K)[0, 0, 0]
    assert s2[a] == s2[b]
    lo, hi = min(a, b), max(a, b)
    n_better = sum(1 for i in range(S, L - W) if s2[i] > s2[a])
    if n_better == k - 1:
        assert lo in sel and hi not in sel
    assert kept[0, 0].tolist() == list(range(S)) + brute_topk(s2, S, W, k) + list(range(L - W, L))


@pytest.mark.parametrize("mode", [GROUP_SUM, PER_QUERY])
def test_partition_invariants(ref, mode):
    P, Hq, Hkv, d, L, S, W, k = 1, 6, 2, 16, 300, 5, 17, 40
    q, K, V = rand_inputs(7, P, Hq, Hkv, d, L, BF16)
    G = Hq // Hkv
    nl = 1 if mode == GROUP_SUM else G
    Kc, Vc, kept = ref.select(BF16, mode, q, K, V, S, W, k)
    assert kept.shape[-1] == S + nl * k + W  # Step 3: length S + k + R + 1 per list
    for c in range(Hkv):
        row = kept[0, c]
        assert row[:S].tolist() == list(range(S))  # sink always kept
        assert row[-W:].tolist() == list(range(L - W, L))  # recent + last token always kept
        for g in range(nl):
            seg = row[S + g * k:S + (g + 1) * k]
            assert np.all(np.diff(seg) > 0) and seg.min() >= S and seg.max() < L - W
    # k = 0: exactly StreamingLLM's sink + recent cache
    _, _, kept0 = ref.select(BF16, mode, q, K, V, S, W, 0)
    assert kept0[0, 0].tolist() == list(range(S)) + list(range(L - W, L))
    # k = E, group-sum: nothing evicted, reduced cache is the cache
    if mode == GROUP_SUM:
        KcE, VcE, keptE = ref.select(BF16, mode, q, K, V, S, W, L - S - W)
        assert keptE[0, 1].tolist() == list(range(L))
        np.testing.assert_array_equal(KcE, K)
        np.testing.assert_array_equal(VcE, V)


def test_modes_coincide_for_G1_and_per_query_equals_logit_topk(ref):
    q, K, V = rand_inputs(8, 1, 3, 3, 16, 200, BF16)
    a = ref.select(BF16, GROUP_SUM, q, K, V, 4, 8, 30)
    b = ref.select(BF16, PER_QUERY, q, K, V, 4, 8, 30)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    # softmax is monotone: per-query selection = top-k of raw logits (computed by the library)
    q2, K2, V2 = rand_inputs(9, 1, 4, 2, 16, 200, F32)
    _, _, kept = ref.select(F32, PER_QUERY, q2, K2, V2, 4, 8, 30)
    logits = np.einsum("hd,hld->hl", q2[0].astype(np.float64), np.repeat(K2[0].astype(np.float64), 2, axis=0))
    for h in range(4):
        top = np.sort(np.argsort(-logits[h, 4:192], kind="stable")[:30] + 4)
        assert kept[0, h // 2, 4 + (h % 2) * 30:4 + (h % 2 + 1) * 30].tolist() == top.tolist()


def test_rejects_bad_arguments(ref):
    q, K, V = rand_inputs(10, 1, 2, 1, 8, 20, F32)
    with pytest.raises(ValueError):
        ref.select(F32, GROUP_SUM, q, K, V, 4, 8, 9)  # S + W + k > L
    with pytest.raises(ValueError):
        ref.select(F32, GROUP_SUM, q, K, V, 4, 0, 2)  # recent must hold the last token


# ------------------------------------------------------------------ append
@pytest.mark.parametrize("t_steps", [1, 3, 6, 9])
def test_fifo_append(ref, t_steps):
    P, Hkv, d, S, k, W = 2, 2, 8, 2, 3, 6
    cap = S + k + W
    key = synth.stream_key(11, 1)
    Kc = synth.fill_host(key, 0, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d)
    Vc = synth.fill_host(key, 5000, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d)
    K0, V0 = Kc.copy(), Vc.copy()
    news = []
    for t in range(t_steps):
        kn = synth.fill_host(key, 100000 + t * 64, P * Hkv * d, BF16).reshape(P, Hkv, d)
        vn = synth.fill_host(key, 200000 + t * 64, P * Hkv * d, BF16).reshape(P, Hkv, d)
        news.append((kn, vn))
        ref.append(BF16, Kc, Vc, kn, vn, S + k, W)
    # sink and selected untouched; window = last W - t originals then the t new, oldest first
    np.testing.assert_array_equal(Kc[:, :, :S + k], K0[:, :, :S + k])
    np.testing.assert_array_equal(Vc[:, :, :S + k], V0[:, :, :S + k])
    hist_k = [K0[:, :, S + k + i] for i in range(W)] + [n[0] for n in news]
    hist_v = [V0[:, :, S + k + i] for i in range(W)] + [n[1] for n in news]
    for i in range(W):
        np.testing.assert_array_equal(Kc[:, :, S + k + i], hist_k[len(hist_k) - W + i])
        np.testing.assert_array_equal(Vc[:, :, S + k + i], hist_v[len(hist_v) - W + i])


def test_grow_append(ref):
    P, Hkv, d, cap = 1, 2, 8, 10
    Kc = np.zeros((P, Hkv, cap, d), np.float32)
    Vc = np.zeros((P, Hkv, cap, d), np.float32)
    kn = np.ones((P, Hkv, d), np.float32)
    n = ref.append(F32, Kc, Vc, kn, 2 * kn, 0, 0, grow=True, length=7)
    assert n == 8 and Kc[0, 1, 7, 0] == 1 and Vc[0, 0, 7, 3] == 2 and Kc[0, 0, 6].sum() == 0
    with pytest.raises(ValueError):
        ref.append(F32, Kc, Vc, kn, kn, 0, 0, grow=True, length=cap)


# ------------------------------------------------------------------ decode attention
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_decode_equals_library_attention(ref, dtype):
    P, Hq, Hkv, d, n = 2, 6, 2, 16, 37
    q, Kc, Vc = rand_inputs(12, P, Hq, Hkv, d, n + 3, dtype)  # capacity n + 3, only n valid
    out = ref.decode_attn(dtype, GROUP_SUM, q, Kc, Vc, n)
    p = np_probs(q, np.ascontiguousarray(Kc[:, :, :n]), dtype)  # [P,Hq,n]
    V64 = np.repeat(synth.to_f64(Vc[:, :, :n], dtype), Hq // Hkv, axis=1)
    want = np.einsum("phl,phld->phd", p, V64)
    np.testing.assert_allclose(out, want.astype(np.float32), rtol=1e-6, atol=1e-7)


def test_decode_special_cases(ref):
    P, Hq, Hkv, d, n = 1, 4, 2, 8, 12
    q, Kc, Vc = rand_inputs(13, P, Hq, Hkv, d, n, F32)
    # one entry: the output is that value row
    out1 = ref.decode_attn(F32, GROUP_SUM, q, Kc, Vc, 1)
    for h in range(Hq):
        np.testing.assert_array_equal(out1[0, h], Vc[0, h // 2, 0])
    # all keys equal: uniform weights, output = mean of the values
    Kc[:] = Kc[:, :, :1]
    out = ref.decode_attn(F32, GROUP_SUM, q, Kc, Vc, n)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], Vc[0, h // 2].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_nothing_evicted_equals_full_attention(ref, dtype):
    """k = E: decode over the reduced cache must equal plain full attention (independent routine)."""
    P, Hq, Hkv, d, L, S, W = 1, 4, 2, 16, 120, 4, 10
    q, K, V = rand_inputs(14, P, Hq, Hkv, d, L, dtype)
    Kc, Vc, kept = ref.select(dtype, GROUP_SUM, q, K, V, S, W, L - S - W)
    qd = synth.fill_host(synth.stream_key(14, 5), 0, P * Hq * d, dtype).reshape(P, Hq, d)
    out = ref.decode_attn(dtype, GROUP_SUM, qd, Kc, Vc, L)
    for c in range(Hkv):
        full = ref.full_attention(dtype, np.ascontiguousarray(qd[0, 2 * c:2 * c + 2]), K[0, c], V[0, c])
        np.testing.assert_allclose(out[0, 2 * c:2 * c + 2], full, rtol=1e-6, atol=1e-7)


def test_full_attention_matches_library(ref):
    q, K, V = rand_inputs(15, 1, 3, 1, 16, 80, BF16)
    got = ref.full_attention(BF16, np.ascontiguousarray(q[0]), K[0, 0], V[0, 0])
    p = np_probs(q, K, BF16)[0]
    want = p @ synth.to_f64(V[0, 0], BF16)
    np.testing.assert_allclose(got, want.astype(np.float32), rtol=1e-6, atol=1e-7)
    idx = np.array([3, 9, 10, 40, 79])
    got_i = ref.full_attention(BF16, np.ascontiguousarray(q[0]), K[0, 0], V[0, 0], idx)
    p_i = np_probs(q, np.ascontiguousarray(K[:, :, idx]), BF16)[0]
    np.testing.assert_allclose(got_i, (p_i @ synth.to_f64(V[0, 0][idx], BF16)).astype(np.float32), rtol=1e-6,
                               atol=1e-7)


def test_reduced_decode_after_appends_equals_attention_over_surviving_tokens(ref):
    """After t appends the reduced cache holds: sink, selected, the W - t newest original recent
    tokens and the t new ones; decode must equal plain attention over exactly those rows."""
    P, Hq, Hkv, d, L, S, W, k = 1, 4, 2, 16, 90, 3, 6, 12
    q, K, V = rand_inputs(16, P, Hq, Hkv, d, L, F32)
    Kc, Vc, kept = ref.select(F32, GROUP_SUM, q, K, V, S, W, k)
    key = synth.stream_key(16, 9)
    Kext, Vext = [K[0, c].copy() for c in range(Hkv)], [V[0, c].copy() for c in range(Hkv)]
    t_steps = 4
    for t in range(t_steps):
        kn = synth.fill_host(key, t * 100, P * Hkv * d, F32).reshape(P, Hkv, d)
        vn = synth.fill_host(key, 5000 + t * 100, P * Hkv * d, F32).reshape(P, Hkv, d)
        ref.append(F32, Kc, Vc, kn, vn, S + k, W)
        for c in range(Hkv):
            Kext[c] = np.vstack([Kext[c], kn[0, c][None]])
            Vext[c] = np.vstack([Vext[c], vn[0, c][None]])
    qd = synth.fill_host(key, 99999, P * Hq * d, F32).reshape(P, Hq, d)
    out = ref.decode_attn(F32, GROUP_SUM, qd, Kc, Vc, S + k + W)
    for c in range(Hkv):
        idx = kept[0, c, :S + k].tolist() + list(range(L - W + t_steps, L + t_steps))
        full = ref.full_attention(F32, np.ascontiguousarray(qd[0, 2 * c:2 * c + 2]), Kext[c], Vext[c], idx)
        np.testing.assert_allclose(out[0, 2 * c:2 * c + 2], full, rtol=1e-6, atol=1e-7)


def test_per_query_decode_uses_own_list(ref):
    P, Hq, Hkv, d, L, S, W, k = 1, 4, 2, 16, 100, 2, 5, 7
    q, K, V = rand_inputs(17, P, Hq, Hkv, d, L, F32)
    Kc, Vc, kept = ref.select(F32, PER_QUERY, q, K, V, S, W, k)
    out = ref.decode_attn(F32, PER_QUERY, q, Kc, Vc, 0, S, k, W)
    G = 2
    for h in range(Hq):
        c, g = h // G, h % G
        idx = kept[0, c, :S].tolist() + kept[0, c, S + g * k:S + (g + 1) * k].tolist() + kept[0, c, S + G * k:].tolist()
        full = ref.full_attention(F32, np.ascontiguousarray(q[0, h:h + 1]), K[0, c], V[0, c], idx)
        np.testing.assert_allclose(out[0, h], full[0], rtol=1e-6, atol=1e-7)


# ------------------------------------------------------------------ paper's printed values
# ------------------------------------------------------------------ StreamLLM_R (window-relative rotary positions)
def inv_freq_of(d, base=500000.0):
    return base ** (-np.arange(0, d, 2, dtype=np.float64) / d)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_window_rope_equals_the_complex_form_of_rotary_attention(ref, dtype):
    """RoFormer's complex form: with z_j = x[j] + i x[j + d/2], the rotated dot product is
    Re sum_j zq_j conj(zk_j) exp(i theta_j (p_q - p_k)): the logits depend on position DIFFERENCES
    only.  Written with library complex arithmetic, no rotation of either vector."""
    P, Hq, Hkv, d, n = 2, 6, 2, 16, 29
    q, Kc, Vc = rand_inputs(31, P, Hq, Hkv, d, n + 2, dtype)
    f = inv_freq_of(d, 100.0)  # a small base: angles up to ~28 rad, every pair turns visibly
    out = ref.decode_attn_window_rope(dtype, q, Kc, Vc, n, f)
    q64, K64, V64 = (synth.to_f64(x, dtype) for x in (q, Kc, Vc))
    h = d // 2
    zq = q64[..., :h] + 1j * q64[..., h:]
    zk = K64[..., :n, :h] + 1j * K64[..., :n, h:]
    delta = (n - 1) - np.arange(n)                      # p_q - p_k
    turn = np.exp(1j * delta[:, None] * f[None, :])     # [n, h]
    G = Hq // Hkv
    want = np.empty((P, Hq, d))
    for p in range(P):
        for hq in range(Hq):
            logit = np.real((zq[p, hq][None, :] * np.conj(zk[p, hq // G]) * turn).sum(-1)) / math.sqrt(d)
            w = np.exp(logit - logit.max())
            want[p, hq] = (w / w.sum()) @ V64[p, hq // G, :n]
    np.testing.assert_allclose(out, want.astype(np.float32), rtol=2e-6, atol=1e-7)


def test_window_rope_special_cases(ref):
    P, Hq, Hkv, d, n = 1, 4, 2, 8, 12
    q, Kc, Vc = rand_inputs(32, P, Hq, Hkv, d, n, F32)
    # zero frequencies: no rotation at all, plain attention
    plain = ref.decode_attn(F32, GROUP_SUM, q, Kc, Vc, n)
    np.testing.assert_array_equal(ref.decode_attn_window_rope(F32, q, Kc, Vc, n, np.zeros(d // 2)), plain)
    # one entry: query and key share position 0, the output is that value row
    out1 = ref.decode_attn_window_rope(F32, q, Kc, Vc, 1, inv_freq_of(d))
    for h in range(Hq):
        np.testing.assert_array_equal(out1[0, h], Vc[0, h // 2, 0])
    # d = 2, theta = pi/2, q = k = (s, 0): logit(distance D) = s^2 cos(D pi/2) / sqrt(2)
    s_ = 3.0
    q2 = np.array([[[s_, 0.0]]], dtype=np.float32)
    K2 = np.tile(np.array([s_, 0.0], dtype=np.float32), (1, 1, 4, 1))
    V2 = np.eye(4, 2, dtype=np.float32).reshape(1, 1, 4, 2) + np.arange(4, dtype=np.float32).reshape(1, 1, 4, 1)
    out = ref.decode_attn_window_rope(F32, q2, K2, V2, 4, np.array([math.pi / 2]))
    logit = np.array([s_ * s_ * math.cos((3 - i) * math.pi / 2) for i in range(4)]) / math.sqrt(2.0)
    w = np.exp(logit - logit.max())
    np.testing.assert_allclose(out[0, 0], (w / w.sum()) @ V2[0, 0].astype(np.float64), rtol=1e-6)


def test_paper_budget_golden(ref):
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_budget.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for B, G, sink, k, recent in (map(int, r) for r in rows):
        assert ref.paper_budget(B, G) == (sink, k, recent)
        assert sink + G * k + recent == B  # per-query-head lists fill the budget exactly


# ------------------------------------------------------------------ planted needles (config C1)
def test_needles_are_all_selected_on_C1(ref):
    cfg = synth.CONFIGS["C1"]
    q, K, V, pos = synth.kv_host(cfg)
    _, _, kept = ref.select(cfg.dtype, GROUP_SUM, q, K, V, cfg.n_sink, cfg.n_recent, cfg.k)
    kept = kept.reshape(cfg.rows, -1)
    for r in range(cfg.rows):
        assert set(pos[r].tolist()) <= set(kept[r].tolist())
