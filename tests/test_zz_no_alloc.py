"""sagekv_decode_step_static: the decode step for callers that cannot allocate (the split partials
live in a scratch array built into the library).  Through the C ABI, against sagekv_decode_step with
a caller workspace and against the oracle, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
BF16 = synth.BF16


def one_call(ref, sk, torch, P, Hq, Hkv, d, S, k, W, n_appended, seed):
    Bt = S + k + W
    key = synth.stream_key(seed, 66)
    Kc = synth.fill_host(key, 0, P * Hkv * Bt * d, BF16).reshape(P, Hkv, Bt, d)
    Vc = synth.fill_host(key, 1 << 30, P * Hkv * Bt * d, BF16).reshape(P, Hkv, Bt, d)
    q = synth.fill_host(key, 2 << 30, P * Hq * d, BF16).reshape(P, Hq, d)
    kn = synth.fill_host(key, 3 << 30, P * Hkv * d, BF16).reshape(P, Hkv, d)
    vn = synth.fill_host(key, 4 << 30, P * Hkv * d, BF16).reshape(P, Hkv, d)
    Kc_s, Vc_s = synth.host_to_torch(Kc, BF16), synth.host_to_torch(Vc, BF16)
    Kc_w, Vc_w = Kc_s.clone(), Vc_s.clone()
    qd, knd, vnd = (synth.host_to_torch(x, BF16) for x in (q, kn, vn))
    desc, ws, out_w = gu.gpu_decode_setup(BF16, P, Hq, Hkv, d, S, k, W, Bt)
    assert 0 < sk.sagekv_decode_workspace_bytes(desc) <= sk.binding.STATIC_SCRATCH_BYTES  # rows are sliced: scratch in use
    out_s = torch.full_like(out_w, float("nan"))
    sk.sagekv_decode_step_static(desc, qd, knd, vnd, Kc_s, Vc_s, n_appended, out_s)
    sk.sagekv_decode_step(desc, qd, knd, vnd, Kc_w, Vc_w, n_appended, out_w, ws)
    torch.cuda.synchronize()
    # the oracle's FIFO keeps the window in age order; n_appended tokens went in before, so rotate
    # the window to the state the ring has: the slot the new token takes holds the oldest entry
    base = S + k
    order = [(n_appended + j) % W for j in range(W)]
    Kc[:, :, base:] = Kc[:, :, base:][:, :, order]
    Vc[:, :, base:] = Vc[:, :, base:][:, :, order]
    ref.append(BF16, Kc, Vc, kn, vn, base, W)
    want = ref.decode_attn(BF16, 0, q, Kc, Vc, Bt)
    got = out_s.cpu().numpy()
    err = np.abs(got - want).max()
    assert err <= gu.DECODE_ATOL[BF16], f"abs err {err:.3e} against the oracle"
    assert torch.equal(out_s, out_w), "differs from sagekv_decode_step with a caller workspace"
    assert torch.equal(Kc_s, Kc_w) and torch.equal(Vc_s, Vc_w)


def test_static_scratch_step_twice_second_call_smaller(ref):
    import torch

    import paper_2503_08879_amd as sk

    one_call(ref, sk, torch, 4, 8, 2, 128, 4, 3580, 512, 7, seed=1201)     # 8 rows x 4096 tokens (one Llama layer)
    one_call(ref, sk, torch, 1, 14, 2, 128, 4, 700, 64, 70, seed=1202)     # smaller, G = 7, window wrapped


def test_static_scratch_rejects_what_does_not_fit():
    import torch

    import paper_2503_08879_amd as sk

    # 160 rows x 13 slices x 16 heads x (128 + 2) floats is more than the built-in 4 MiB
    P, Hq, Hkv, d, S, k, W = 80, 32, 2, 128, 4, 20000, 64
    desc = sk.decode_desc(P, Hq, Hkv, d, sk.BF16, S, k, W, S + k + W)
    assert sk.sagekv_decode_workspace_bytes(desc) > sk.binding.STATIC_SCRATCH_BYTES
    z = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    out = torch.full((16,), -7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(sk.SagekvError) as e:
        sk.sagekv_decode_step_static(desc, z, z, z, z, z, 0, out)  # rejected on the host: nothing is read or written
    assert e.value.code == sk.binding.ERR_SCRATCH_LIMIT
    assert "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.max()) == -7.0
