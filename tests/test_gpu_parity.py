"""HIP path vs CPU oracle, element by element, through the C-ABI binding.  Needs an MI355X."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

BF16, F32 = synth.BF16, synth.F32
GROUP_SUM = 0


def rand_case(seed, P, Hq, Hkv, d, L, dtype):
    key = synth.stream_key(seed, 55)
    q = synth.fill_host(key, 0, P * Hq * d, dtype).reshape(P, Hq, d)
    K = synth.fill_host(key, 1 << 30, P * Hkv * L * d, dtype).reshape(P, Hkv, L, d)
    V = synth.fill_host(key, 1 << 32, P * Hkv * L * d, dtype).reshape(P, Hkv, L, d)
    return q, K, V


def select_parity(ref, dtype, q, K, V, S, W, k, cap=None):
    """Both routes of sagekv_select against the oracle: with scores_out (dense path, scores checked
    too) and without (pre-filtered path wherever it applies).  Returns the second run's outputs."""
    Kc, Vc, kept, s = ref.select(dtype, GROUP_SUM, q, K, V, S, W, k, cap, want_scores=True)
    for want_scores in (True, False):
        out = gu.gpu_select(dtype, q, K, V, S, W, k, cap, want_scores=want_scores)
        if want_scores:
            gu.check_scores(out["scores"], s[:, :, 0])
        n_ex = gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k)
        gu.check_gather(out, K, V, S, k, W)
        if n_ex == 0:
            np.testing.assert_array_equal(out["Kc"], Kc)
            np.testing.assert_array_equal(out["Vc"], Vc)
    return out, (Kc, Vc, kept, s)


# ----------------------------------------------------------------------------- generator
def test_device_fill_equals_host_fill():
    import torch

    for dtype, td in ((BF16, torch.bfloat16), (F32, torch.float32)):
        key = synth.stream_key(4242, synth.T_K)
        t = torch.empty(100_003, dtype=td, device="cuda")
        synth.fill_device(t, key, 0)
        np.testing.assert_array_equal(synth.torch_to_host(t, dtype), synth.fill_host(key, 0, 100_003, dtype))
        t2 = torch.empty(4096, dtype=td, device="cuda")
        synth.fill_device(t2, key, 12345 * 8)
        np.testing.assert_array_equal(synth.torch_to_host(t2, dtype), synth.fill_host(key, 12345 * 8, 4096, dtype))


def test_device_config_equals_host_config():
    cfg = synth.CONFIGS["C1"]
    q, K, V, pos = synth.kv_host(cfg)
    qd, Kd, Vd, pos_d = synth.kv_device(cfg)
    np.testing.assert_array_equal(synth.torch_to_host(Kd, cfg.dtype), K)
    np.testing.assert_array_equal(synth.torch_to_host(Vd, cfg.dtype), V)
    np.testing.assert_array_equal(synth.torch_to_host(qd, cfg.dtype), q)


# ----------------------------------------------------------------------------- select
def test_select_C1(ref):
    cfg = synth.CONFIGS["C1"]
    q, K, V, pos = synth.kv_host(cfg)
    out, _ = select_parity(ref, cfg.dtype, q, K, V, cfg.n_sink, cfg.n_recent, cfg.k)
    kept = out["kept"].reshape(cfg.rows, -1)
    for r in range(cfg.rows):
        assert set(pos[r].tolist()) <= set(kept[r].tolist())  # every needle survives


@pytest.mark.parametrize(
    "dtype,Hq,Hkv,d,L,S,W,k",
    [
        (BF16, 8, 2, 128, 5037, 4, 64, 300),     # G=4, ragged L (not a multiple of any tile)
        (BF16, 7, 1, 128, 9001, 3, 17, 500),     # G=7 (Qwen group), odd everything
        (BF16, 4, 4, 64, 4100, 0, 1, 100),       # G=1, d=64, no sink, window = last token only
        (F32, 6, 2, 128, 3000, 5, 40, 123),      # fp32, d=128, G=3
        (F32, 4, 2, 64, 1025, 4, 16, 64),        # fp32, d=64
        (BF16, 16, 2, 128, 2050, 2, 30, 77),     # G=8
        (BF16, 20, 2, 128, 1500, 2, 30, 77),     # G=10: two score launches per row
    ],
)
def test_select_shapes(ref, dtype, Hq, Hkv, d, L, S, W, k):
    q, K, V = rand_case(100 + Hq + L, 2, Hq, Hkv, d, L, dtype)
    select_parity(ref, dtype, q, K, V, S, W, k, cap=S + k + W + 5)


@pytest.mark.parametrize("k_kind", ["zero", "one", "E-1", "E"])
def test_select_k_extremes(ref, k_kind):
    P, Hq, Hkv, d, L, S, W = 1, 8, 2, 128, 1300, 4, 20
    E = L - S - W
    k = {"zero": 0, "one": 1, "E-1": E - 1, "E": E}[k_kind]
    q, K, V = rand_case(7, P, Hq, Hkv, d, L, BF16)
    out, _ = select_parity(ref, BF16, q, K, V, S, W, k)
    if k_kind == "E":
        np.testing.assert_array_equal(out["Kc"], K)  # nothing evicted: the reduced cache IS the cache
        np.testing.assert_array_equal(out["Vc"], V)
    if k_kind == "zero":
        assert out["kept"][0, 0].tolist() == list(range(S)) + list(range(L - W, L))


def test_select_no_candidates(ref):
    q, K, V = rand_case(8, 1, 4, 2, 64, 40, F32)
    select_parity(ref, F32, q, K, V, 8, 32, 0)  # E = 0


def test_select_tiny_rows_at_every_alignment(ref):
    """Few candidates, every offset of the candidate range against the 16-byte loads of the dense
    top-k (first candidate S = 0..3 floats into its score row, 1..9 candidates, odd row pitches)."""
    for S in range(4):
        for E in (1, 2, 3, 4, 5, 6, 7, 8, 9):
            W = 2 + (S + E) % 3
            L = S + E + W
            q, K, V = rand_case(300 + 10 * S + E, 2, 4, 2, 64, L, F32)
            for k in sorted({1, (E + 1) // 2, E}):
                select_parity(ref, F32, q, K, V, S, W, k)


def test_select_ties_at_every_alignment(ref):
    """q = 0 makes every score equal, so the dense top-k takes its general route (exact radix select,
    count-then-write compaction by wave-owned segments) and must hand the ties to the lowest indices,
    at every offset of the candidate range against its 16-byte loads and with ragged ends."""
    for S in range(4):
        for E in (5, 9, 300, 5003):
            W = 3 + (S + E) % 2
            L = S + E + W
            q, K, V = rand_case(400 + 10 * S + E % 7, 1, 4, 2, 64, L, BF16)
            q[:] = 0
            for k in sorted({1, E // 2, E - 1}):
                for want_scores in (True, False):
                    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=want_scores)
                    want = list(range(S + k)) + list(range(L - W, L))
                    for c in range(2):
                        assert out["kept"][0, c].tolist() == want, (S, E, k, want_scores)


def test_select_row_longer_than_the_lds_bitmap(ref):
    """More than 512K candidates: the dense top-k writes its output with the two-pass route."""
    P, Hq, Hkv, d, L, S, W, k = 1, 2, 1, 64, 540001, 3, 50, 2000
    q, K, V = rand_case(11, P, Hq, Hkv, d, L, BF16)
    select_parity(ref, BF16, q, K, V, S, W, k)


def test_prefiltered_path_at_a_million_tokens(ref):
    """L = 1,000,000: the longest rows the pre-filtered path takes (one bit per candidate in LDS)."""
    P, Hq, Hkv, d, L, S, W, k = 1, 8, 2, 128, 1_000_000, 4, 1024, 7164
    q, K, V = rand_case(1_000_003, P, Hq, Hkv, d, L, BF16)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False)
    assert out["redone"] == 0  # certified by the pre-filtered path, not redone densely
    if gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k) == 0:
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)
    # per-query lists at the same length
    kq = 1024
    Kc, Vc, kept, s = ref.select(BF16, 1, q, K, V, S, W, kq, want_scores=True)
    out = gu.gpu_select(BF16, q, K, V, S, W, kq, want_scores=False, head_mode=1)
    assert out["redone"] == 0
    G = Hq // Hkv
    for g in range(G):
        got = np.concatenate([out["kept"][:, :, :S], out["kept"][:, :, S + g * kq:S + (g + 1) * kq], out["kept"][:, :, S + G * kq:]], axis=2)
        want = np.concatenate([kept[:, :, :S], kept[:, :, S + g * kq:S + (g + 1) * kq], kept[:, :, S + G * kq:]], axis=2)
        gu.check_kept(got, want, s[:, :, g], S, W, kq)


def test_select_all_scores_equal_takes_lowest_indices(ref):
    """q = 0: every probability is 1/L, the whole row ties; the first k candidates must win."""
    P, Hq, Hkv, d, L, S, W, k = 1, 8, 2, 128, 6000, 4, 50, 700
    q, K, V = rand_case(9, P, Hq, Hkv, d, L, BF16)
    q[:] = 0
    out = gu.gpu_select(BF16, q, K, V, S, W, k)
    want = list(range(S + k)) + list(range(L - W, L))
    for c in range(Hkv):
        assert out["kept"][0, c].tolist() == want
    select_parity(ref, BF16, q, K, V, S, W, k)


def test_select_duplicate_keys_straddling_the_threshold(ref):
    """Copies of the k-th best key have exactly its score; only the lowest indices may be kept."""
    P, Hq, Hkv, d, L, S, W, k = 1, 4, 1, 128, 3000, 4, 20, 200
    q, K, V = rand_case(10, P, Hq, Hkv, d, L, BF16)
    s = ref.scores(BF16, GROUP_SUM, q, K)[0, 0, 0]
    order = sorted(range(S, L - W), key=lambda i: (-float(s[i]), i))
    kth = order[k - 1]
    for j in (S, 1000, 1001, 2500, L - W - 1):  # plant copies, incl. first and last candidate
        if j != kth:
            K[0, 0, j] = K[0, 0, kth]
    select_parity(ref, BF16, q, K, V, S, W, k)


def test_select_strided_token_major_layout(ref):
    """K, V stored [P, L, Hkv, d] (token-major) and passed through the stride fields."""
    import torch

    P, Hq, Hkv, d, L, S, W, k = 2, 8, 2, 128, 2000, 4, 32, 150
    q, K, V = rand_case(11, P, Hq, Hkv, d, L, BF16)
    Kd = synth.host_to_torch(np.ascontiguousarray(K.transpose(0, 2, 1, 3)), BF16).permute(0, 2, 1, 3)
    Vd = synth.host_to_torch(np.ascontiguousarray(V.transpose(0, 2, 1, 3)), BF16).permute(0, 2, 1, 3)
    assert not Kd.is_contiguous()
    out = gu.gpu_select(BF16, q, None, None, S, W, k, K_dev=Kd, V_dev=Vd)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    assert gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k) == 0
    np.testing.assert_array_equal(out["Kc"], Kc)
    np.testing.assert_array_equal(out["Vc"], Vc)


def test_select_is_deterministic():
    q, K, V = rand_case(12, 2, 8, 2, 128, 20000, BF16)
    first = gu.gpu_select(BF16, q, K, V, 4, 128, 1000)
    for _ in range(4):
        again = gu.gpu_select(BF16, q, K, V, 4, 128, 1000)
        for name in ("kept", "Kc", "Vc", "scores"):
            np.testing.assert_array_equal(first[name], again[name])


def test_select_without_scores_out_matches(ref):
    q, K, V = rand_case(13, 1, 8, 2, 128, 4099, BF16)
    a = gu.gpu_select(BF16, q, K, V, 4, 64, 256, want_scores=True)
    b = gu.gpu_select(BF16, q, K, V, 4, 64, 256, want_scores=False)
    np.testing.assert_array_equal(a["kept"], b["kept"])
    np.testing.assert_array_equal(a["Kc"], b["Kc"])


@pytest.mark.parametrize(
    "Hq,Hkv,d,L,S,W,k",
    [
        (8, 2, 128, 40000, 4, 128, 1000),    # G=4
        (7, 1, 128, 50021, 3, 77, 2000),     # G=7, ragged
        (16, 2, 128, 30011, 0, 1, 500),      # G=8, no sink, window = last token
        (24, 2, 128, 24000, 4, 64, 300),     # G=12: heads padded to 16
        (4, 2, 64, 33000, 4, 300, 800),      # d=64, G=2
        (3, 3, 64, 20000, 70, 400, 1),       # G=1, k=1, sink and window larger than their samples
    ],
)
def test_select_prefiltered_path(ref, Hq, Hkv, d, L, S, W, k):
    """Shapes where the pre-filtered path applies (bf16, 5k + 8192 <= E): it must certify its rows."""
    q, K, V = rand_case(200 + Hq + d, 2, Hq, Hkv, d, L, BF16)
    out, _ = select_parity(ref, BF16, q, K, V, S, W, k)
    assert out["redone"] == 0
    dense = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False, flags=1)
    assert dense["redone"] == -1
    np.testing.assert_array_equal(dense["kept"], out["kept"])


def test_prefilter_falls_back_when_all_scores_tie(ref):
    """q = 0: every token passes the filter, the candidate list overflows, every row is redone densely."""
    P, Hq, Hkv, d, L, S, W, k = 1, 8, 2, 128, 30000, 4, 50, 700
    q, K, V = rand_case(9, P, Hq, Hkv, d, L, BF16)
    q[:] = 0
    out, _ = select_parity(ref, BF16, q, K, V, S, W, k)
    assert out["redone"] == P * Hkv
    want = list(range(S + k)) + list(range(L - W, L))
    for c in range(Hkv):
        assert out["kept"][0, c].tolist() == want


def test_prefilter_falls_back_for_more_rows_than_a_gated_launch_has_row_blocks(ref):
    """20 rows that all tie: the gated dense stages loop over the flagged rows inside their workgroups."""
    P, Hq, Hkv, d, L, S, W, k = 10, 8, 2, 64, 20000, 3, 40, 400
    q, K, V = rand_case(12, P, Hq, Hkv, d, L, BF16)
    q[:] = 0
    q[7] = rand_case(13, 1, Hq, Hkv, d, 8, BF16)[0][0]   # one problem with ordinary scores in between
    out, _ = select_parity(ref, BF16, q, K, V, S, W, k)
    assert out["redone"] == (P - 1) * Hkv
    want = list(range(S + k)) + list(range(L - W, L))
    for pr in range(P):
        if pr != 7:
            for c in range(Hkv):
                assert out["kept"][pr, c].tolist() == want


@pytest.mark.parametrize("sampled", [True, False])
def test_prefilter_with_one_token_carrying_most_of_the_mass(ref, sampled):
    """One candidate holds ~70% of head 0's attention.  Scaled up by the sampling rate it would make
    the sampled normaliser ~40 times too large; the sampler counts a token that would stand for more
    than 1 % of a head's mass once, so the row is certified whether the sample contains the token or
    misses it (then the filter is merely more permissive).  Either way the result is exact."""
    P, Hq, Hkv, d, L, S, W, k = 1, 4, 1, 128, 40000, 4, 64, 500
    q, K, V = rand_case(21, P, Hq, Hkv, d, L, BF16)
    E = L - S - W
    n_runs = 4 * max(16, min(128, E // 4096))  # the library samples this many 16-token runs of candidates
    start7 = S + ((7 * (((E - 16) << 16) // (n_runs - 1))) >> 16)
    t = start7 + 5 + (0 if sampled else 300)  # inside sampled run 7, or between runs 7 and 8
    q64 = synth.to_f64(q[0, 0], BF16)
    K[0, 0, t] = synth.round_to_dtype(12.0 * q64 / np.linalg.norm(q64), BF16)  # logit ~ 12
    out, _ = select_parity(ref, BF16, q, K, V, S, W, k)
    assert out["redone"] == 0
    assert t in out["kept"][0, 0].tolist()


@pytest.mark.parametrize("scale,share", [(2.5, 0.1), (4.0, 0.4)])
def test_prefilter_certifies_heavy_tailed_attention(ref, scale, share):
    """Queries scaled so that the logits have a standard deviation of ~2.5 (~4): the 100 heaviest of
    65536 tokens hold a quarter (two thirds) of a head's attention, as in a trained model.  Heavy sampled
    tokens are counted once and a row that shows them takes a lower threshold; without either, one such
    row in seven (three) could not be certified."""
    P, Hq, Hkv, d, L, S, W, k = 2, 16, 4, 128, 65536, 4, 256, 1788
    q, K, V = rand_case(77, P, Hq, Hkv, d, L, BF16)
    q = synth.round_to_dtype(scale * synth.to_f64(q, BF16), BF16)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    top100 = np.sort(s[0, 0, 0].astype(np.float64))[::-1][:100].sum() / Hq * Hkv
    assert top100 > share, top100  # share of the 4 heads' summed mass held by 100 tokens
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False)
    assert out["redone"] == 0
    n_ex = gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k)
    if n_ex == 0:
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)


def test_prefilter_certifies_model_like_attention(ref):
    """An attention profile shaped like a trained model's: eight very heavy first tokens (four of them
    outside the sink, among the candidates), a recent window with an exponential bump, a heavy-tailed
    middle.  The pre-filtered path must certify every row and agree with the oracle."""
    P, Hq, Hkv, d, L, S, W, k = 1, 8, 2, 128, 65536, 4, 256, 1788
    G = Hq // Hkv
    q, K, V = rand_case(78, P, Hq, Hkv, d, L, BF16)
    q64 = 2.5 * synth.to_f64(q, BF16)
    q = synth.round_to_dtype(q64, BF16)
    K64 = synth.to_f64(K, BF16)
    qdir = q64.reshape(P, Hkv, G, d).mean(2)
    qdir /= np.linalg.norm(qdir, axis=-1, keepdims=True)
    boost = np.zeros(L)
    boost[:8] = 10.0
    t = np.arange(L - 2048, L)
    boost[t] += 4.0 * np.exp(-(L - 1 - t) / 512.0)
    unit = np.sqrt(G) / 2.5   # key displacement along qdir for about one unit of logit
    K64 += boost[None, None, :, None] * unit * qdir[:, :, None, :]
    K = synth.round_to_dtype(K64, BF16)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    row = s[0, 0, 0].astype(np.float64)
    assert row[:8].sum() / G > 0.05 and row[L - W:].sum() / G > 0.01  # the profile is what it says
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False)
    assert out["redone"] == 0
    n_ex = gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k)
    assert set(range(4, 8)) <= set(out["kept"][0, 0].tolist())  # the heavy candidates are kept
    if n_ex == 0:
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)


def far_down_case(seed, P, Hq, Hkv, d, L, scale):
    """Queries scaled so that the logits have a standard deviation of about `scale`."""
    q, K, V = rand_case(seed, P, Hq, Hkv, d, L, BF16)
    return synth.round_to_dtype(scale * synth.to_f64(q, BF16), BF16), K, V


def check_far_down(ref, head_mode, q, K, V, S, W, k, route, min_far):
    """Kept sets and gathered rows against the oracle where the k-th score lies under fp32's normal
    range (2^-126): the oracle ranks the fp32-rounded scores, denormals included, and exact zeros by
    index.  route: 'scores' (dense, scores_out given), 'dense' (flag) or 'auto' (pre-filtered where it applies)."""
    P, Hq, d = q.shape
    Hkv, L = K.shape[1], K.shape[2]
    G = Hq // Hkv if head_mode == 1 else 1
    Kc, Vc, kept, s = ref.select(BF16, head_mode, q, K, V, S, W, k, want_scores=True)  # s [P,Hkv,lists,L]
    tiny = np.float32(2.0 ** -126)
    cand = s[..., S:L - W]
    kth = np.sort(cand, axis=-1)[..., ::-1][..., k - 1]
    assert (kth < tiny).mean() >= min_far, f"only {(kth < tiny).mean():.2f} of the lists have a k-th score under 2^-126"
    assert ((cand < tiny) & (cand > 0)).any(), "no denormal score in the case"
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=route == "scores", flags=1 if route == "dense" else 0,
                        head_mode=head_mode)
    if route == "scores":
        # fp32 logits carry an absolute error that grows with their size (~|logit| 2^-24 times a few), so do
        # the scores relative to their size; below 2^-126 they sit on the 2^-149 grid, each head's term rounded to it
        g, w = out["scores"].reshape(s.shape).astype(np.float64), s.astype(np.float64)
        assert np.all(np.abs(g - w) <= 1e-3 * w + (Hq // Hkv + 1) * 2.0 ** -149)
    for li in range(G):
        cut = lambda a: np.concatenate([a[..., :S], a[..., S + li * k:S + (li + 1) * k], a[..., S + G * k:]], axis=-1)
        got, want = cut(out["kept"]), cut(kept)
        if not np.array_equal(got, want):
            assert (kth[:, :, li] > 0).all(), "kept sets differ where the k-th score is an exact zero (ties go by index)"
            gu.check_kept(got, want, s[:, :, li], S, W, k)
    if np.array_equal(out["kept"], kept):
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)
    return out


@pytest.mark.parametrize("head_mode", [0, 1])
@pytest.mark.parametrize("route", ["scores", "dense"])
@pytest.mark.parametrize("k_kind", ["E/8", "E/4", "E/2", "E-1"])
def test_select_ranks_scores_below_the_normal_range_dense(ref, head_mode, route, k_kind):
    """Logits spread over +-150: most candidates sit more than 100 logits below their row maximum,
    where exp() leaves fp32's normal range.  The selection must still follow the oracle: denormal
    scores by value, exact zeros by index."""
    P, Hq, Hkv, d, L, S, W = 2, 8, 2, 128, 5200, 4, 40
    E = L - S - W
    k = {"E/8": E // 8, "E/4": E // 4, "E/2": E // 2, "E-1": E - 1}[k_kind]
    q, K, V = far_down_case(500, P, Hq, Hkv, d, L, 40.0)
    check_far_down(ref, head_mode, q, K, V, S, W, k, route, min_far=1.0 if k_kind in ("E/2", "E-1") else 0.0)


@pytest.mark.parametrize("head_mode", [0, 1])
@pytest.mark.parametrize("scale,k", [(40.0, 2500), (50.0, 3000), (55.0, 4000), (70.0, 2000)])
def test_select_ranks_scores_below_the_normal_range_prefiltered(ref, head_mode, scale, k):
    """The same regime on a row long enough for the pre-filtered path (5 k lists <= E): whether it can
    certify such a row or hands it to the dense path, the kept set is the oracle's."""
    P, Hq, Hkv, d, L, S, W = 1, 4, 2, 128, 60000, 4, 64
    q, K, V = far_down_case(501, P, Hq, Hkv, d, L, scale)
    out = check_far_down(ref, head_mode, q, K, V, S, W, k, "auto", min_far=0.5 if scale > 50 else 0.0)
    assert out["redone"] >= 0  # the call went through the pre-filtered path


@pytest.mark.parametrize("route", ["prefiltered", "two_sweeps", "one_sweep"])
def test_group_sum_order_when_few_tokens_hold_a_heads_mass(ref, route):
    """Queries scaled by 9: one token holds 50-98 % of each head's softmax, with a logit of about 36.
    An fp32 logit of that size is off by ~1e-5, and so would be a normaliser summed from fp32 logits;
    the two heads of a group would be off by different amounts, enough to swap group-sum scores that
    are 2e-6 apart (this case did, at token 145332 of row 1).  The kernels take such terms with an fp64
    exponent; every route must give the oracle's kept set."""
    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, L, S, W, k = 1, 4, 2, 128, 162963, 300, 1, 26083
    key = synth.stream_key(880000 + 3879, 55)
    q = synth.fill_host(key, 0, P * Hq * d, BF16).reshape(P, Hq, d)
    q = synth.round_to_dtype(9.0 * synth.to_f64(q, BF16), BF16)
    K = synth.fill_host(key, 1 << 30, P * Hkv * L * d, BF16).reshape(P, Hkv, L, d)
    V = synth.fill_host(key, 1 << 33, P * Hkv * L * d, BF16).reshape(P, Hkv, L, d)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=route == "two_sweeps",
                        flags=sk.SELECT_DENSE if route == "one_sweep" else 0)
    assert (out["redone"] >= 0) == (route == "prefiltered")
    assert gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k) == 0  # no near-tie exemption needed here
    np.testing.assert_array_equal(out["Kc"], Kc)


def test_prefilter_chunk_slots_overflow_into_the_row_pool(ref):
    """Every score chunk owns a few candidate slots; here the heavy tokens all sit in two chunks (as the
    tokens next to the recent window do in a trained model), far more than those chunks' own slots hold,
    so most candidates go through the row's overflow pool.  The kept set is still the oracle's and the
    rows are certified without the dense stages."""
    P, Hq, Hkv, d, L, S, W, k = 1, 8, 2, 128, 40000, 4, 128, 1000
    G = Hq // Hkv
    q, K, V = rand_case(91, P, Hq, Hkv, d, L, BF16)
    q64 = synth.to_f64(q, BF16)
    K64 = synth.to_f64(K, BF16)
    qdir = q64.reshape(P, Hkv, G, d).mean(2)
    qdir /= np.linalg.norm(qdir, axis=-1, keepdims=True)
    # tokens 37000 .. 38799 (chunks 36 and 37 of 1024 tokens): +3 logits or so on every head of the group
    K64[:, :, 37000:38800] += 3.0 * np.sqrt(G) * qdir[:, :, None, :]
    K = synth.round_to_dtype(K64, BF16)
    Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, q, K, V, S, W, k, want_scores=True)
    inside = ((kept[0, :, S:S + k] >= 37000) & (kept[0, :, S:S + k] < 38800)).sum(axis=-1)
    assert (inside > 700).all(), inside  # the selection is mostly that cluster: 350 tokens a chunk against 64-128 slots
    out = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False)
    assert out["redone"] == 0
    n_ex = gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k)
    if n_ex == 0:
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)


def test_scores_out_without_the_dense_flag_takes_two_sweeps(ref):
    """A call that asks for every score on a descriptor the pre-filtered path serves has no logit scratch:
    it reads K twice (softmax statistics, then scores).  Scores and kept sets as the oracle's, and as
    the one-sweep dense path's (flag) kept set."""
    for head_mode in (0, 1):
        P, Hq, Hkv, d, L, S, W, k = 2, 14, 2, 128, 33001, 3, 70, 400
        q, K, V = rand_case(92 + head_mode, P, Hq, Hkv, d, L, BF16)
        G = Hq // Hkv if head_mode else 1
        Kc, Vc, kept, s = ref.select(BF16, head_mode, q, K, V, S, W, k, want_scores=True)
        two = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=True, head_mode=head_mode)
        one = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=True, head_mode=head_mode, flags=1)
        assert two["redone"] == -1 and one["redone"] == -1
        for out in (two, one):
            gu.check_scores(out["scores"].reshape(s.shape), s)
            for li in range(G):
                cut = lambda a: np.concatenate([a[..., :S], a[..., S + li * k:S + (li + 1) * k], a[..., S + G * k:]], axis=-1)
                gu.check_kept(cut(out["kept"]), cut(kept), s[:, :, li], S, W, k)
        np.testing.assert_array_equal(two["kept"], one["kept"])


def test_select_C2_shape_two_layers(ref):
    """Config C2's row shape (32q/8kv, d128, bf16, L 32768, 4+1788+256) on 2 of its 32 layers."""
    cfg = synth.CONFIGS["C2"].with_(n_layers=2)
    q, K, V, pos = synth.kv_host(cfg)
    out, _ = select_parity(ref, cfg.dtype, q, K, V, cfg.n_sink, cfg.n_recent, cfg.k)
    assert out["redone"] == 0
    kept = out["kept"].reshape(cfg.rows, -1)
    for r in range(cfg.rows):
        assert set(pos[r].tolist()) <= set(kept[r].tolist())


def test_layer_by_layer_on_two_streams_equals_one_batched_call():
    """Per-layer streaming: the pass of layer l is enqueued on a side stream as soon as that layer's
    cache exists (its own workspace per stream), while the caller goes on; results are those of one
    call over all layers."""
    import torch

    import paper_2503_08879_amd as sk

    layers, Hq, Hkv, d, L, S, W, k = 6, 8, 2, 128, 36000, 4, 128, 700
    q, K, V = rand_case(321, layers, Hq, Hkv, d, L, BF16)
    whole = gu.gpu_select(BF16, q, K, V, S, W, k, want_scores=False)
    assert whole["redone"] == 0
    qd, Kd, Vd = (synth.host_to_torch(x, BF16) for x in (q, K, V))
    Bt = S + k + W
    Kc = torch.zeros((layers, Hkv, Bt, d), dtype=qd.dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.zeros((layers, Hkv, Bt), dtype=torch.int32, device="cuda")
    desc = sk.select_desc(qd[:1], Kd[:1], Vd[:1], S, W, k, Bt)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda") for _ in streams]
    torch.cuda.synchronize()
    for l in range(layers):
        with torch.cuda.stream(streams[l % 2]):
            sl = slice(l, l + 1)
            sk.sagekv_select(desc, qd[sl], Kd[sl], Vd[sl], Kc[sl], Vc[sl], kept[sl], None, wss[l % 2])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kept.cpu().numpy(), whole["kept"])
    np.testing.assert_array_equal(synth.torch_to_host(Kc, BF16), whole["Kc"])
    np.testing.assert_array_equal(synth.torch_to_host(Vc, BF16), whole["Vc"])


def test_prefiltered_select_is_deterministic():
    """The candidate lists are filled in whatever order the workgroups run; the result must not depend on it."""
    q, K, V = rand_case(14, 2, 8, 2, 128, 40000, BF16)
    first = gu.gpu_select(BF16, q, K, V, 4, 128, 1000, want_scores=False)
    assert first["redone"] == 0
    for _ in range(4):
        again = gu.gpu_select(BF16, q, K, V, 4, 128, 1000, want_scores=False)
        for name in ("kept", "Kc", "Vc"):
            np.testing.assert_array_equal(first[name], again[name])


def test_refresh_reselect_on_a_grown_cache(ref):
    """Interval refresh (the paper's future work, Sec. 4): the full cache is kept in a buffer with
    spare capacity, generated tokens are appended to it, and the eviction pass is run again with the
    current token's query over the longer prefix, into the same reduced cache."""
    import torch

    P, Hq, Hkv, d, L0, Lcap, S, W, k = 1, 8, 2, 128, 30000, 30100, 4, 64, 600
    q, K, V = rand_case(15, P, Hq, Hkv, d, Lcap, BF16)
    Kd, Vd = synth.host_to_torch(K, BF16), synth.host_to_torch(V, BF16)
    prev = None
    for L in (L0, L0 + 37, Lcap):  # prefill, then two refreshes after 37 and 100 generated tokens
        qL = synth.fill_host(synth.stream_key(15, 9), L, P * Hq * d, BF16).reshape(P, Hq, d)
        out = gu.gpu_select(BF16, qL, None, None, S, W, k, want_scores=False, K_dev=Kd[:, :, :L], V_dev=Vd[:, :, :L])
        Kc, Vc, kept, s = ref.select(BF16, GROUP_SUM, qL, np.ascontiguousarray(K[:, :, :L]),
                                     np.ascontiguousarray(V[:, :, :L]), S, W, k, want_scores=True)
        assert gu.check_kept(out["kept"], kept, s[:, :, 0], S, W, k) == 0
        np.testing.assert_array_equal(out["Kc"], Kc)
        np.testing.assert_array_equal(out["Vc"], Vc)
        assert prev is None or not np.array_equal(prev, out["kept"])
        prev = out["kept"]


# ----------------------------------------------------------------------------- error paths (host checks only)
def test_invalid_arguments_are_rejected_before_launch():
    import torch

    import paper_2503_08879_amd as sk

    q = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((1, 2, 512, 128), dtype=torch.bfloat16, device="cuda")
    kept = torch.full((1, 2, 100), -7, dtype=torch.int32, device="cuda")
    Kc = torch.zeros((1, 2, 100, 128), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")

    def call(desc, ws_=ws):
        sk.sagekv_select(desc, q, K, K, Kc, Kc, kept, None, ws_)

    good = sk.select_desc(q, K, K, 4, 32, 64, 100)
    call(good)
    for field, value, code in [("k", 600, 1), ("n_recent", 0, 1), ("compact_capacity", 50, 1), ("n_q_heads", 3, 1),
                               ("head_dim", 96, 2), ("dtype", 5, 2), ("head_mode", 7, 1), ("k_stride_token", 100, 2)]:
        bad = sk.select_desc(q, K, K, 4, 32, 64, 100)
        setattr(bad, field, value)
        kept.fill_(-7)
        with pytest.raises(sk.SagekvError) as e:
            call(bad)
        assert e.value.code == code, field
        assert sk.sagekv_select_workspace_bytes(bad) == 0
        torch.cuda.synchronize()
        assert int(kept.max()) == -7  # nothing written
    with pytest.raises(sk.SagekvError) as e:
        call(good, ws[:1024])
    assert e.value.code == 3
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_select(good, q, None, K, Kc, Kc, kept, None, ws)  # null required pointer
    assert e.value.code == 1
    flat = torch.zeros(K.numel() + 8, dtype=torch.bfloat16, device="cuda")
    K_off = flat[1:1 + K.numel()].view(K.shape)  # same strides, base pointer 2 bytes off a 16-byte boundary
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_select(good, q, K_off, K, Kc, Kc, kept, None, ws)
    assert e.value.code == 2

    # decode calls
    dd = sk.decode_desc(1, 4, 2, 128, sk.BF16, 4, 64, 32, 100)
    dws = torch.empty(max(sk.sagekv_decode_workspace_bytes(dd), 16), dtype=torch.uint8, device="cuda")
    out = torch.full((1, 4, 128), -7.0, dtype=torch.float32, device="cuda")
    kn = torch.zeros((1, 2, 128), dtype=torch.bfloat16, device="cuda")
    sk.sagekv_decode_step(dd, q, kn, kn, Kc, Kc.clone(), 0, out, dws)
    torch.cuda.synchronize()
    out.fill_(-7.0)

    def code_of(fn):
        try:
            fn()
        except sk.SagekvError as e:
            return e.code
        return 0

    assert code_of(lambda: sk.sagekv_decode_attn(dd, q, Kc, Kc, 0, out, dws)) == 1            # len < 1
    assert code_of(lambda: sk.sagekv_decode_attn(dd, q, Kc, Kc, 101, out, dws)) == 1          # len > capacity
    assert code_of(lambda: sk.sagekv_decode_attn(dd, None, Kc, Kc, 10, out, dws)) == 1        # null query
    q_off = torch.zeros(q.numel() + 8, dtype=torch.bfloat16, device="cuda")[3:3 + q.numel()].view(q.shape)
    assert code_of(lambda: sk.sagekv_decode_attn(dd, q_off, Kc, Kc, 10, out, dws)) == 2       # misaligned query
    assert code_of(lambda: sk.sagekv_decode_attn_window(dd, q, None, Kc, Kc, 10, out, dws)) == 1   # null sink query
    assert code_of(lambda: sk.sagekv_decode_step(dd, q, kn, kn, Kc, Kc, -1, out, dws)) == 1   # negative counter
    long_row = sk.decode_desc(1, 4, 2, 128, sk.BF16, 4, 900, 32, 1000)  # long enough to be split: needs scratch
    Kl = torch.zeros((1, 2, 1000, 128), dtype=torch.bfloat16, device="cuda")
    assert sk.sagekv_decode_workspace_bytes(long_row) > 8
    assert code_of(lambda: sk.sagekv_decode_step(long_row, q, kn, kn, Kl, Kl, 0, out, dws[:8])) == 3  # too small
    assert code_of(lambda: sk.sagekv_decode_step(long_row, q, kn, kn, Kl, Kl, 0, out, None)) == 3     # missing
    grow = sk.decode_desc(1, 4, 2, 128, sk.BF16, 4, 64, 32, 100, True)
    assert code_of(lambda: sk.sagekv_decode_step(grow, q, kn, kn, Kc, Kc, 0, out, dws)) == 1  # grown row exceeds capacity
    bad = sk.decode_desc(1, 4, 2, 96, sk.BF16, 4, 64, 32, 100)
    assert code_of(lambda: sk.sagekv_decode_attn(bad, q, Kc, Kc, 10, out, dws)) == 2          # head_dim
    torch.cuda.synchronize()
    assert float(out.max()) == -7.0  # nothing written


def test_many_rows_in_one_call(ref):
    """64000 rows of a short cache in one call (the largest row counts a call takes: rows index a grid
    dimension): the eviction pass against the oracle on every row, then decode steps on the reduced cache."""
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, L, S, W, k = 8000, 8, 8, 64, 72, 2, 6, 9
    q, K, V = rand_case(31337, P, Hq, Hkv, d, L, BF16)
    out, (Kc_r, Vc_r, kept_r, s_r) = select_parity(ref, BF16, q, K, V, S, W, k)
    Bt = S + k + W
    # decode is compared where the kept sets are identical (all rows, but for a near-tie swap the contract allows)
    same = (out["kept"] == kept_r).reshape(P, -1).all(axis=1)
    assert same.mean() > 0.999
    ddesc = sk.decode_desc(P, Hq, Hkv, d, BF16, S, k, W, Bt)
    dws = torch.empty(max(sk.sagekv_decode_workspace_bytes(ddesc), 16), dtype=torch.uint8, device="cuda")
    res = torch.empty((P, Hq, d), dtype=torch.float32, device="cuda")
    key = synth.stream_key(31338, 7)
    for t in range(W + 1):  # once around the recent ring
        qs = synth.fill_host(key, t * 3 << 24, P * Hq * d, BF16).reshape(P, Hq, d)
        kn = synth.fill_host(key, (t * 3 + 1) << 24, P * Hkv * d, BF16).reshape(P, Hkv, d)
        vn = synth.fill_host(key, (t * 3 + 2) << 24, P * Hkv * d, BF16).reshape(P, Hkv, d)
        sk.sagekv_decode_step(ddesc, *(synth.host_to_torch(x, BF16) for x in (qs, kn, vn)), out["Kc_dev"], out["Vc_dev"],
                              t, res, dws)
        torch.cuda.synchronize()
        ref.append(BF16, Kc_r, Vc_r, kn, vn, S + k, W)
        want = ref.decode_attn(BF16, GROUP_SUM, qs, Kc_r, Vc_r, Bt)
        assert np.abs(res.cpu().numpy() - want)[same].max() <= gu.DECODE_ATOL[BF16], f"step {t}"


def test_row_limit_is_reported():
    """More than 65535 rows (or selection lists) in one call: SAGEKV_ERR_UNSUPPORTED before any launch."""
    import torch

    import paper_2503_08879_amd as sk

    P, Hkv, d, L = 8192, 8, 64, 16  # 65536 rows
    q = torch.zeros((P, Hkv, d), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((P, Hkv, L, d), dtype=torch.bfloat16, device="cuda")
    Kc = torch.zeros((P, Hkv, 8, d), dtype=torch.bfloat16, device="cuda")
    kept = torch.full((P, Hkv, 8), -7, dtype=torch.int32, device="cuda")
    desc = sk.select_desc(q, K, K, 2, 2, 4, 8)
    assert sk.sagekv_select_workspace_bytes(desc) == 0
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_select(desc, q, K, K, Kc, Kc, kept, None, ws)
    assert e.value.code == 2
    ddesc = sk.decode_desc(P, Hkv, Hkv, d, sk.BF16, 2, 4, 2, 8)
    out = torch.full((P, Hkv, d), -7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_decode_attn(ddesc, q, Kc, Kc, 8, out, ws)
    assert e.value.code == 2
    # 16384 rows of 4 per-query lists each are as many lists
    q4 = torch.zeros((2048, 4 * Hkv, d), dtype=torch.bfloat16, device="cuda")
    d4 = sk.select_desc(q4, K[:2048], K[:2048], 2, 2, 1, 8, head_mode=sk.PER_QUERY)
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_select(d4, q4, K[:2048], K[:2048], Kc[:2048], Kc[:2048], kept[:2048], None, ws)
    assert e.value.code == 2
    torch.cuda.synchronize()
    assert int(kept.max()) == -7 and float(out.max()) == -7.0  # nothing written


# ----------------------------------------------------------------------------- decode
def decode_case(ref, dtype, P, Hq, Hkv, d, S, k, W, steps, seed, grow=False, fused=True, q_scale=1.0):
    import torch

    import paper_2503_08879_amd as sk

    Bt = S + k + W
    cap = Bt + (steps if grow else 3)
    key = synth.stream_key(seed, 66)
    Kc = synth.fill_host(key, 0, P * Hkv * cap * d, dtype).reshape(P, Hkv, cap, d)
    Vc = synth.fill_host(key, 1 << 30, P * Hkv * cap * d, dtype).reshape(P, Hkv, cap, d)
    Kc_d, Vc_d = synth.host_to_torch(Kc, dtype), synth.host_to_torch(Vc, dtype)
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, cap, grow)
    length = Bt
    worst = 0.0
    for t in range(steps):
        q = synth.fill_host(key, (2 << 30) + t * 10_000_000, P * Hq * d, dtype).reshape(P, Hq, d)
        if q_scale != 1.0:  # peaked attention: logits of magnitude ~4 q_scale
            q = synth.round_to_dtype(q_scale * synth.to_f64(q, dtype), dtype)
        kn = synth.fill_host(key, (3 << 30) + t * 10_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        vn = synth.fill_host(key, (4 << 30) + t * 10_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        length = ref.append(dtype, Kc, Vc, kn, vn, S + k, W, grow=grow, length=length)
        want = ref.decode_attn(dtype, GROUP_SUM, q, Kc, Vc, length)
        qd, knd, vnd = (synth.host_to_torch(x, dtype) for x in (q, kn, vn))
        if fused:
            sk.sagekv_decode_step(desc, qd, knd, vnd, Kc_d, Vc_d, t, out, ws)
        else:
            sk.sagekv_append(desc, knd, vnd, Kc_d, Vc_d, t)
            sk.sagekv_decode_attn(desc, qd, Kc_d, Vc_d, length, out, ws)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy() - want).max()
        worst = max(worst, float(err))
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: abs err {err:.3e}"
    # the physical cache holds the same multiset of rows as the oracle's shifted one
    got_K = synth.torch_to_host(Kc_d, dtype)
    np.testing.assert_array_equal(got_K[:, :, :S + k], Kc[:, :, :S + k])
    if not grow:
        for p in range(P):
            for c in range(Hkv):
                a = sorted(map(bytes, got_K[p, c, S + k:Bt]))
                b = sorted(map(bytes, Kc[p, c, S + k:Bt]))
                assert a == b
    else:
        np.testing.assert_array_equal(got_K[:, :, :length], Kc[:, :, :length])
    return worst


@pytest.mark.parametrize(
    "dtype,Hq,Hkv,d,S,k,W,steps",
    [
        (F32, 4, 2, 64, 4, 188, 64, 8),      # config C1's decode shape
        (BF16, 8, 2, 128, 4, 300, 33, 40),   # window wraps around (steps > W)
        (BF16, 7, 1, 128, 4, 500, 64, 5),    # G=7
        (BF16, 4, 4, 64, 0, 90, 5, 7),       # G=1, d=64, no sink
        (F32, 6, 2, 128, 2, 100, 9, 12),     # fp32 d=128
        (BF16, 20, 2, 128, 4, 200, 16, 3),   # G=10: heads padded to 16
        (BF16, 16, 1, 128, 4, 200, 16, 3),   # G=16: a full tile of heads
        (BF16, 40, 2, 64, 4, 200, 16, 3),    # G=20: two launches per step (16 + 4), d=64
    ],
)
def test_decode_steps_fused(ref, dtype, Hq, Hkv, d, S, k, W, steps):
    decode_case(ref, dtype, 2, Hq, Hkv, d, S, k, W, steps, seed=20 + Hq)


@pytest.mark.parametrize(
    "rows,Hq,Hkv,d,S,k,W",
    [
        (200, 8, 2, 128, 4, 250, 47),     # G=4
        (200, 14, 2, 128, 4, 250, 47),    # G=7
        (200, 24, 2, 128, 3, 130, 30),    # G=12
        (200, 16, 1, 64, 4, 250, 47),     # G=16, d=64
        (200, 3, 3, 64, 0, 100, 33),      # G=1
        (300, 14, 2, 128, 4, 250, 47),    # more rows than CUs, G=7: 4-wave workgroups
        (300, 8, 2, 128, 4, 250, 47),     # more rows than CUs, G=4
    ],
)
def test_decode_one_workgroup_per_row(ref, rows, Hq, Hkv, d, S, k, W):
    """192 rows or more: every row is one workgroup's, no merge launch (the layout of a whole
    model's decode step)."""
    P = -(-rows // Hkv)
    decode_case(ref, BF16, P, Hq, Hkv, d, S, k, W, 3, seed=60 + Hq)


@pytest.mark.parametrize("dtype", [BF16, F32])
@pytest.mark.parametrize("q_scale", [9.0, 40.0])
@pytest.mark.parametrize("rows,Hq,Hkv", [(3, 8, 2), (200, 4, 1)])
def test_decode_with_peaked_attention(ref, dtype, q_scale, rows, Hq, Hkv):
    """Scaled queries: logits of magnitude up to ~170, one token holds nearly all of a head's attention.
    The stated tolerances hold there too (fp32 caches: the kernel takes its logits in fp64)."""
    decode_case(ref, dtype, max(1, rows // Hkv), Hq, Hkv, 128, 4, 1500, 64, 3, seed=515, q_scale=q_scale)


def test_decode_steps_separate_append(ref):
    decode_case(ref, BF16, 2, 8, 2, 128, 4, 300, 33, 6, seed=31, fused=False)


def test_decode_grow_mode(ref):
    decode_case(ref, BF16, 1, 8, 2, 128, 4, 100, 16, 6, seed=32, grow=True)
    decode_case(ref, F32, 1, 4, 2, 64, 4, 100, 16, 4, seed=33, grow=True, fused=False)


def test_decode_len_one_and_long_rows(ref):
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, cap = 3, 8, 2, 128, 9000
    key = synth.stream_key(40, 66)
    Kc = synth.fill_host(key, 0, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d)
    Vc = synth.fill_host(key, 1 << 30, P * Hkv * cap * d, BF16).reshape(P, Hkv, cap, d)
    q = synth.fill_host(key, 2 << 30, P * Hq * d, BF16).reshape(P, Hq, d)
    desc, ws, out = gu.gpu_decode_setup(BF16, P, Hq, Hkv, d, 4, cap - 4 - 8, 8, cap)
    Kd, Vd, qd = (synth.host_to_torch(x, BF16) for x in (Kc, Vc, q))
    for length in (1, 2, 63, 64, 65, 4097, cap):
        sk.sagekv_decode_attn(desc, qd, Kd, Vd, length, out, ws)
        torch.cuda.synchronize()
        want = ref.decode_attn(BF16, GROUP_SUM, q, Kc, Vc, length)
        assert np.abs(out.cpu().numpy() - want).max() <= gu.DECODE_ATOL[BF16], length
    sk.sagekv_decode_attn(desc, qd, Kd, Vd, 1, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for h in range(Hq):  # one entry: the output is that value row, exactly
        np.testing.assert_array_equal(got[:, h], synth.to_f64(Vc[:, h // 4, 0], BF16).astype(np.float32))


def test_nothing_evicted_equals_full_attention_end_to_end(ref):
    """k = E: select then decode over the reduced cache equals plain attention over the full cache."""
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, L, S, W = 1, 8, 2, 128, 3000, 4, 40
    q, K, V = rand_case(50, P, Hq, Hkv, d, L, BF16)
    out = gu.gpu_select(BF16, q, K, V, S, W, L - S - W)
    desc, ws, o = gu.gpu_decode_setup(BF16, P, Hq, Hkv, d, S, L - S - W, W, L)
    qd = synth.host_to_torch(q, BF16)
    sk.sagekv_decode_attn(desc, qd, out["Kc_dev"], out["Vc_dev"], L, o, ws)
    torch.cuda.synchronize()
    got = o.cpu().numpy()
    for c in range(Hkv):
        full = ref.full_attention(BF16, np.ascontiguousarray(q[0, 4 * c:4 * c + 4]), K[0, c], V[0, c])
        assert np.abs(got[0, 4 * c:4 * c + 4] - full).max() <= gu.DECODE_ATOL[BF16]


def test_C1_end_to_end(ref):
    """Config C1: select, then 8 decode steps with the config's seeded q / k_new / v_new."""
    import torch

    import paper_2503_08879_amd as sk

    cfg = synth.CONFIGS["C1"]
    q, K, V, _ = synth.kv_host(cfg)
    S, W, k = cfg.n_sink, cfg.n_recent, cfg.k
    out = gu.gpu_select(cfg.dtype, q, K, V, S, W, k)
    Kc, Vc, kept = ref.select(cfg.dtype, GROUP_SUM, q, K, V, S, W, k)
    np.testing.assert_array_equal(out["kept"], kept)
    desc, ws, o = gu.gpu_decode_setup(cfg.dtype, cfg.n_problems, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, S, k, W,
                                      cfg.budget)
    for t in range(cfg.decode_steps):
        qs, kn, vn = synth.decode_inputs_host(cfg, t)
        ref.append(cfg.dtype, Kc, Vc, kn, vn, S + k, W)
        want = ref.decode_attn(cfg.dtype, GROUP_SUM, qs, Kc, Vc, cfg.budget)
        qd, knd, vnd = (synth.host_to_torch(x, cfg.dtype) for x in (qs, kn, vn))
        sk.sagekv_decode_step(desc, qd, knd, vnd, out["Kc_dev"], out["Vc_dev"], t, o, ws)
        torch.cuda.synchronize()
        assert np.abs(o.cpu().numpy() - want).max() <= gu.DECODE_ATOL[cfg.dtype]


# ----------------------------------------------------------------------------- per-query head mode (paper-literal)
def per_query_case(ref, dtype, P, Hq, Hkv, d, L, S, W, k, steps, seed, expect_fast=None):
    """Select with one top-k per query head, then decode steps where head g attends sink + its own
    list + recent (Sec. 2 Step 2, App. A.2)."""
    import torch

    import paper_2503_08879_amd as sk

    G = Hq // Hkv
    q, K, V = rand_case(seed, P, Hq, Hkv, d, L, dtype)
    dense = gu.gpu_select(dtype, q, K, V, S, W, k, head_mode=1)
    Kc, Vc, kept, s = ref.select(dtype, 1, q, K, V, S, W, k, want_scores=True)  # s [P,Hkv,G,L]
    gu.check_scores(dense["scores"].reshape(P, Hkv, G, L), s)
    out = gu.gpu_select(dtype, q, K, V, S, W, k, head_mode=1, want_scores=False)  # pre-filtered where it applies
    if expect_fast is not None:
        assert (out["redone"] == 0) == expect_fast, out["redone"]
    if np.array_equal(dense["kept"], kept):
        np.testing.assert_array_equal(out["kept"], dense["kept"])
    n_kept = S + G * k + W
    assert out["kept"].shape[-1] == n_kept
    n_ex = 0
    for g in range(G):  # every list against the oracle's, with the near-tie exemption
        sub_gpu = np.concatenate([out["kept"][..., :S], out["kept"][..., S + g * k:S + (g + 1) * k],
                                  out["kept"][..., S + G * k:]], axis=-1)
        sub_ref = np.concatenate([kept[..., :S], kept[..., S + g * k:S + (g + 1) * k], kept[..., S + G * k:]], axis=-1)
        n_ex += gu.check_kept(sub_gpu, sub_ref, s[:, :, g], S, W, k)
    gu.check_gather(out, K, V, S, G * k, W)
    if n_ex:
        return
    np.testing.assert_array_equal(out["Kc"], Kc)
    np.testing.assert_array_equal(out["Vc"], Vc)
    desc, ws, o = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, n_kept, head_mode=1)
    key = synth.stream_key(seed, 91)
    for t in range(steps):
        qs = synth.fill_host(key, t * 1_000_000, P * Hq * d, dtype).reshape(P, Hq, d)
        kn = synth.fill_host(key, (1 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        vn = synth.fill_host(key, (2 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        ref.append(dtype, Kc, Vc, kn, vn, S + G * k, W)
        want = ref.decode_attn(dtype, 1, qs, Kc, Vc, 0, S, k, W)
        sk.sagekv_decode_step(desc, *(synth.host_to_torch(x, dtype) for x in (qs, kn, vn)), out["Kc_dev"],
                              out["Vc_dev"], t, o, ws)
        torch.cuda.synchronize()
        err = np.abs(o.cpu().numpy() - want).max()
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: {err:.3e}"


@pytest.mark.parametrize(
    "dtype,P,Hq,Hkv,d,L,S,W,k,steps",
    [
        (F32, 1, 4, 2, 64, 4096, 4, 64, 94, 8),        # config C1 with k = 94 per query head
        (BF16, 2, 8, 2, 128, 6000, 16, 40, 150, 45),   # G=4, window wraps
        (BF16, 1, 7, 1, 128, 5000, 3, 17, 99, 4),      # G=7
        (BF16, 3, 4, 4, 64, 3000, 0, 1, 50, 3),        # G=1: same as group-sum
        (F32, 1, 6, 2, 128, 2000, 5, 33, 0, 3),        # k = 0
        (BF16, 100, 14, 2, 128, 1500, 8, 32, 40, 2),   # 200 rows, G=7: one workgroup per row in decode
        (BF16, 150, 8, 2, 128, 1200, 8, 32, 40, 2),    # 300 rows, G=4
    ],
)
def test_per_query_mode(ref, dtype, P, Hq, Hkv, d, L, S, W, k, steps):
    per_query_case(ref, dtype, P, Hq, Hkv, d, L, S, W, k, steps, seed=300 + Hq + d)


def test_per_query_paper_budget(ref):
    """The appendix's split for Llama (B = 8192, G = 4): sink 2048, 1024 per query head, recent 2048,
    on a 32K-token bf16 cache of two Llama-shaped layers."""
    sink, k, recent = ref.paper_budget(8192, 4)
    per_query_case(ref, BF16, 2, 32, 8, 128, 32768, sink, recent, k, 2, seed=77, expect_fast=True)


def test_per_query_prefiltered_G7(ref):
    """Qwen-shaped group (G = 7) with the appendix's split of B = 8192 (2048 / 7 x 512 / 2560)."""
    sink, k, recent = ref.paper_budget(8192, 7)
    per_query_case(ref, BF16, 1, 14, 2, 128, 50000, sink, recent, k, 2, seed=78, expect_fast=True)
