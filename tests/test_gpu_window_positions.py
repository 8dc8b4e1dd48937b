"""StreamLLM_R cache mode (Sec. 3.1 baseline (3a), App. A.1): window-relative rotary positions.

The oracle follows the description literally: an un-rotated cache, every entry rotated at its
window index, the query at the last index.  The HIP path keeps the usual cache (keys rotated
once, at their absolute positions) and is given two rotations of the query; rotary attention
depends on position differences only, so both must agree.  The rotations that feed the HIP path
are the model's job, done here in numpy (fp64, rounded to the cache type), independent of the
oracle's C code."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
BF16, F32 = synth.BF16, synth.F32


def rope(x64, pos, inv_freq):
    """Rotary embedding of x64 [..., d] at integer positions pos (broadcast over the leading axes)."""
    h = x64.shape[-1] // 2
    ang = np.asarray(pos, dtype=np.float64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = x64[..., :h], x64[..., h:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def window_case(ref, dtype, P, Hq, Hkv, d, S, W, steps, L0, seed, base=500000.0):
    import torch

    import paper_2503_08879_amd as sk

    n = S + W
    inv_freq = base ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    key = synth.stream_key(seed, 44)
    K_pre = synth.fill_host(key, 0, P * Hkv * n * d, dtype).reshape(P, Hkv, n, d)   # window order, un-rotated
    V = synth.fill_host(key, 1 << 30, P * Hkv * n * d, dtype).reshape(P, Hkv, n, d)
    abs_pos = np.concatenate([np.arange(S), np.arange(L0 - W, L0)])                # where the entries came from
    K_abs = synth.round_to_dtype(rope(synth.to_f64(K_pre, dtype), abs_pos, inv_freq), dtype)
    Kc_d, Vc_d = synth.host_to_torch(K_abs, dtype), synth.host_to_torch(V, dtype)
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, 0, W, n)
    worst = 0.0
    for t in range(steps):
        q_pre = synth.fill_host(key, (2 << 30) + t * 1_000_000, P * Hq * d, dtype).reshape(P, Hq, d)
        kn_pre = synth.fill_host(key, (3 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        vn = synth.fill_host(key, (4 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        # oracle: the paper's description
        ref.append(dtype, K_pre, V, kn_pre, vn, S, W)
        want = ref.decode_attn_window_rope(dtype, q_pre, K_pre, V, n, inv_freq)
        # HIP path: the usual rotated cache, two rotations of the query
        now = L0 + t
        q64 = synth.to_f64(q_pre, dtype)
        q_abs = synth.round_to_dtype(rope(q64, now, inv_freq), dtype)
        q_sink = synth.round_to_dtype(rope(q64, n - 1, inv_freq), dtype)
        kn_abs = synth.round_to_dtype(rope(synth.to_f64(kn_pre, dtype), now, inv_freq), dtype)
        args = [synth.host_to_torch(x, dtype) for x in (q_abs, q_sink, kn_abs, vn)]
        sk.sagekv_decode_step_window(desc, *args, Kc_d, Vc_d, t, out, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        err = np.abs(got - want).max()
        worst = max(worst, float(err))
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: abs err {err:.3e}"
        if t == 0 and S >= 20:
            # the sink query matters: with q in its place the result is visibly different
            sk.sagekv_decode_attn_window(desc, args[0], args[0], Kc_d, Vc_d, n, out, ws)
            torch.cuda.synchronize()
            assert np.abs(out.cpu().numpy() - want).max() > 2e-3
    return worst


@pytest.mark.parametrize(
    "dtype,P,Hq,Hkv,d,S,W,steps",
    [
        (F32, 2, 4, 2, 64, 4, 60, 5),         # vector-ALU kernel, split rows
        (F32, 1, 8, 2, 128, 37, 200, 3),      # sink not a multiple of the block
        (BF16, 2, 8, 2, 128, 4, 508, 6),      # MFMA kernel, G = 4
        (BF16, 3, 14, 2, 128, 50, 300, 4),    # G = 7: 16-token blocks, sink ends inside a block
        (BF16, 200, 4, 1, 64, 128, 384, 3),   # many rows: one workgroup per row
        (BF16, 1, 4, 2, 64, 0, 100, 2),       # no sink: both queries unused/used consistently
    ],
)
def test_streamllm_r_equals_rotated_cache_with_two_queries(ref, dtype, P, Hq, Hkv, d, S, W, steps):
    window_case(ref, dtype, P, Hq, Hkv, d, S, W, steps, L0=5000 + 17 * S, seed=P + d + S)


def test_sink_query_equal_to_query_is_plain_attention(ref):
    """q_sink = q: the window call must be the plain call, bit for bit."""
    import torch

    import paper_2503_08879_amd as sk

    dtype, P, Hq, Hkv, d, S, W = BF16, 4, 8, 2, 128, 20, 300
    n = S + W
    key = synth.stream_key(5, 45)
    Kc = synth.host_to_torch(synth.fill_host(key, 0, P * Hkv * n * d, dtype).reshape(P, Hkv, n, d), dtype)
    Vc = synth.host_to_torch(synth.fill_host(key, 1 << 30, P * Hkv * n * d, dtype).reshape(P, Hkv, n, d), dtype)
    q = synth.host_to_torch(synth.fill_host(key, 2 << 30, P * Hq * d, dtype).reshape(P, Hq, d), dtype)
    desc, ws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, 0, W, n)
    out2 = torch.empty_like(out)
    sk.sagekv_decode_attn(desc, q, Kc, Vc, n, out, ws)
    sk.sagekv_decode_attn_window(desc, q, q, Kc, Vc, n, out2, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
