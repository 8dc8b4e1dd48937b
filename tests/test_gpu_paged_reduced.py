"""The reduced cache in pages (block table + page pools), as a serving engine keeps it: the eviction
pass gathers into pages, the decode step stores the new token in the page that holds its ring slot and
attends through the block table.  The layout only says where a token lives, so the oracle runs on the
logical (dense) reduced cache.  Pool pages that no row owns and the tail of a row's last page hold NaN
patterns: a read outside the logical cache would poison the output, a write outside it is detected."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu
from tests.test_gpu_parity import rand_case

pytestmark = pytest.mark.gpu
BF16, F32 = synth.BF16, synth.F32


def nan_of(dtype):
    return np.uint16(0x7FC1) if dtype == BF16 else np.float32(np.nan)


def fresh_pools(P, Hkv, d, cap, page_size, dtype, seed, spare=5):
    """Shuffled block table [P, pages per row] and NaN-filled K / V pools [n_pages, Hkv, page, d]."""
    per = -(-cap // page_size)
    n_pages = P * per + spare
    table = np.random.default_rng(seed).permutation(n_pages)[: P * per].astype(np.int32).reshape(P, per)
    pool = np.full((n_pages, Hkv, page_size, d), nan_of(dtype), dtype=synth.np_dtype(dtype))
    return table, pool, pool.copy(), n_pages


def logical(pool_h, table, n_tokens, page_size):
    """Pool [n_pages,Hkv,page,d] -> logical reduced cache [P,Hkv,n_tokens,d]."""
    P = table.shape[0]
    out = np.empty((P, pool_h.shape[1], n_tokens, pool_h.shape[3]), dtype=pool_h.dtype)
    for p in range(P):
        for j in range(-(-n_tokens // page_size)):
            t0, t1 = j * page_size, min((j + 1) * page_size, n_tokens)
            out[p, :, t0:t1] = pool_h[table[p, j], :, : t1 - t0]
    return out


def untouched_outside(pool_h, table, n_tokens, page_size, dtype):
    """Everything outside the rows' first n_tokens tokens still holds the NaN pattern."""
    mask = np.ones(pool_h.shape[:3], dtype=bool)  # [n_pages, Hkv, page]
    for p in range(table.shape[0]):
        for j in range(table.shape[1]):
            t0 = j * page_size
            mask[table[p, j], :, : max(0, min(page_size, n_tokens - t0))] = False
    rest = pool_h[mask]
    return bool(np.all(rest.view(np.uint16) == 0x7FC1)) if dtype == BF16 else bool(np.all(np.isnan(rest)))


@pytest.mark.parametrize(
    "dtype,P,Hq,Hkv,d,L,S,W,k,page_size,head_mode,steps",
    [
        (BF16, 2, 8, 2, 128, 9000, 4, 40, 700, 16, 0, 90),     # few rows: sliced rows; window wraps twice
        (BF16, 2, 8, 2, 128, 9000, 4, 40, 700, 256, 0, 5),     # pages larger than the window
        (BF16, 100, 8, 2, 128, 1500, 4, 33, 150, 64, 0, 70),   # 200 rows, one workgroup each
        (BF16, 2, 14, 2, 128, 6000, 3, 20, 99, 32, 1, 45),     # per-query lists, G = 7
        (BF16, 1, 4, 4, 64, 3000, 0, 5, 90, 16, 0, 12),        # d = 64, no sink
        (F32, 2, 6, 2, 128, 2000, 5, 17, 123, 16, 0, 40),      # fp32 kernels
    ],
)
def test_select_into_pages_then_paged_decode(ref, dtype, P, Hq, Hkv, d, L, S, W, k, page_size, head_mode, steps):
    import torch

    import paper_2503_08879_amd as sk

    G = Hq // Hkv
    lists = G if head_mode == 1 else 1
    base = S + lists * k
    Bt = base + W
    q, K, V = rand_case(700 + Hq + page_size, P, Hq, Hkv, d, L, dtype)
    table, Kpool, Vpool, n_pages = fresh_pools(P, Hkv, d, Bt, page_size, dtype, seed=Hq + page_size)
    Kp, Vp = synth.host_to_torch(Kpool, dtype), synth.host_to_torch(Vpool, dtype)
    tab = torch.from_numpy(table).cuda()
    qd, Kd, Vd = (synth.host_to_torch(x, dtype) for x in (q, K, V))
    sdesc = sk.select_desc(qd, Kd, Vd, S, W, k, Bt, head_mode=head_mode)
    pages = sk.compact_pages(tab, Kp, Vp)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(sdesc), dtype=torch.uint8, device="cuda")
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    sk.sagekv_select_into_pages(sdesc, None, pages, qd, Kd, Vd, Kp, Vp, kept, None, ws)
    torch.cuda.synchronize()

    Kc_r, Vc_r, kept_r, s_r = ref.select(dtype, head_mode, q, K, V, S, W, k, want_scores=True)
    got = kept.cpu().numpy()
    n_ex = 0
    for li in range(lists):
        cut = lambda a: np.concatenate([a[..., :S], a[..., S + li * k:S + (li + 1) * k], a[..., base:]], axis=-1)
        n_ex += gu.check_kept(cut(got), cut(kept_r), s_r[:, :, li], S, W, k)
    assert n_ex == 0
    Kh, Vh = synth.torch_to_host(Kp, dtype), synth.torch_to_host(Vp, dtype)
    np.testing.assert_array_equal(logical(Kh, table, Bt, page_size), Kc_r)
    np.testing.assert_array_equal(logical(Vh, table, Bt, page_size), Vc_r)
    assert untouched_outside(Kh, table, Bt, page_size, dtype) and untouched_outside(Vh, table, Bt, page_size, dtype)

    # decode steps through the block table: host-counted steps, then the device-counted form
    ddesc, dws, out = gu.gpu_decode_setup(dtype, P, Hq, Hkv, d, S, k, W, Bt, head_mode=head_mode)
    ring = torch.zeros(2, dtype=torch.int32, device="cuda")
    key = synth.stream_key(800 + Hq, 91)
    for t in range(steps):
        qs = synth.fill_host(key, t * 1_000_000, P * Hq * d, dtype).reshape(P, Hq, d)
        kn = synth.fill_host(key, (1 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        vn = synth.fill_host(key, (2 << 30) + t * 1_000_000, P * Hkv * d, dtype).reshape(P, Hkv, d)
        ref.append(dtype, Kc_r, Vc_r, kn, vn, base, W)
        want = ref.decode_attn(dtype, head_mode, qs, Kc_r, Vc_r, Bt, S, k, W)
        ins = [synth.host_to_torch(x, dtype) for x in (qs, kn, vn)]
        if t < steps // 2:
            sk.sagekv_decode_step_paged(ddesc, pages, *ins, Kp, Vp, t, None, out, dws)
            ring.fill_(t + 1)
            ring[1] = 0
        else:
            sk.sagekv_decode_step_paged(ddesc, pages, *ins, Kp, Vp, -1, ring, out, dws)
        torch.cuda.synchronize()
        err = np.abs(out.cpu().numpy() - want).max()
        assert err <= gu.DECODE_ATOL[dtype], f"step {t}: abs err {err:.3e}"
    assert ring.tolist() == [steps, 0]
    # attention alone over a prefix of the paged rows (the ring is not in age order: the oracle gets
    # the pages' own logical content)
    if head_mode == 0:
        n = base + W // 2
        sk.sagekv_decode_attn_paged(ddesc, pages, ins[0], Kp, Vp, n, out, dws)
        torch.cuda.synchronize()
        Kl = np.ascontiguousarray(logical(synth.torch_to_host(Kp, dtype), table, Bt, page_size))
        Vl = np.ascontiguousarray(logical(synth.torch_to_host(Vp, dtype), table, Bt, page_size))
        want = ref.decode_attn(dtype, 0, qs, Kl, Vl, n)
        assert np.abs(out.cpu().numpy() - want).max() <= gu.DECODE_ATOL[dtype]
    # the pages hold the same rows as the oracle's cache (window as a multiset), nothing outside was written
    Kh, Vh = synth.torch_to_host(Kp, dtype), synth.torch_to_host(Vp, dtype)
    Kl = logical(Kh, table, Bt, page_size)
    np.testing.assert_array_equal(Kl[:, :, :base], Kc_r[:, :, :base])
    for p in range(P):
        for c in range(Hkv):
            assert sorted(map(bytes, Kl[p, c, base:])) == sorted(map(bytes, Kc_r[p, c, base:]))
    assert untouched_outside(Kh, table, Bt, page_size, dtype) and untouched_outside(Vh, table, Bt, page_size, dtype)


def test_paged_input_into_paged_reduced_cache(ref):
    """Both caches in pages: full cache read through its block table, reduced cache written through its own."""
    import torch

    import paper_2503_08879_amd as sk
    from tests.test_gpu_paged import to_pages

    dtype, P, Hq, Hkv, d, L, S, W, k, ps_in, ps_out = BF16, 2, 8, 2, 128, 40000, 4, 128, 1000, 64, 32
    Bt = S + k + W
    q, K, V = rand_case(731, P, Hq, Hkv, d, L, dtype)
    per = -(-L // ps_in)
    n_in = P * per + 3
    tab_in = np.random.default_rng(5).permutation(n_in)[: P * per].astype(np.int32).reshape(P, per)
    Kin = synth.host_to_torch(to_pages(K, ps_in, tab_in, n_in, False, dtype), dtype)
    Vin = synth.host_to_torch(to_pages(V, ps_in, tab_in, n_in, False, dtype), dtype)
    table, Kpool, Vpool, _ = fresh_pools(P, Hkv, d, Bt, ps_out, dtype, seed=6)
    Kp, Vp = synth.host_to_torch(Kpool, dtype), synth.host_to_torch(Vpool, dtype)
    qd = synth.host_to_torch(q, dtype)
    tab_in_d, tab_out_d = torch.from_numpy(tab_in).cuda(), torch.from_numpy(table).cuda()  # kept alive: the structs hold pointers
    sdesc, in_pages = sk.paged_select_desc(qd, Kin, Vin, tab_in_d, L, S, W, k, Bt)
    out_pages = sk.compact_pages(tab_out_d, Kp, Vp)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(sdesc), dtype=torch.uint8, device="cuda")
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    sk.sagekv_select_into_pages(sdesc, in_pages, out_pages, qd, Kin, Vin, Kp, Vp, kept, None, ws)
    torch.cuda.synchronize()
    assert sk.sagekv_select_redone_rows(sdesc, ws) == 0
    Kc_r, Vc_r, kept_r = ref.select(dtype, 0, q, K, V, S, W, k)
    np.testing.assert_array_equal(kept.cpu().numpy(), kept_r)
    np.testing.assert_array_equal(logical(synth.torch_to_host(Kp, dtype), table, Bt, ps_out), Kc_r)
    np.testing.assert_array_equal(logical(synth.torch_to_host(Vp, dtype), table, Bt, ps_out), Vc_r)


def test_paged_reduced_cache_arguments_are_checked():
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, S, k, W, ps = 1, 4, 2, 128, 4, 64, 32, 16
    Bt = S + k + W
    pool = torch.zeros((8, Hkv, ps, d), dtype=torch.bfloat16, device="cuda")
    tab = torch.arange(7, dtype=torch.int32, device="cuda").view(1, 7)  # 7 pages x 16 = 112 >= 100 tokens
    z = torch.zeros((P, Hq, d), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((P, Hkv, d), dtype=torch.bfloat16, device="cuda")
    out = torch.full((P, Hq, d), -7.0, dtype=torch.float32, device="cuda")
    dd = sk.decode_desc(P, Hq, Hkv, d, sk.BF16, S, k, W, Bt)
    ws = torch.empty(max(sk.sagekv_decode_workspace_bytes(dd), 16), dtype=torch.uint8, device="cuda")

    def code_of(pages, n=0):
        try:
            sk.sagekv_decode_step_paged(dd, pages, z, kn, kn, pool, pool, n, None, out, ws)
        except sk.SagekvError as e:
            return e.code
        return 0

    good = sk.compact_pages(tab, pool, pool)
    assert code_of(good) == 0
    torch.cuda.synchronize()
    out.fill_(-7.0)
    for field, value, code in [("page_size", 24, 1), ("page_size", 8, 1), ("table_pitch", 6, 1), ("n_pages", 0, 1),
                               ("k_stride_page", Hkv * ps * d - 8, 1), ("v_stride_page", Hkv * ps * d + 4, 2)]:
        bad = sk.compact_pages(tab, pool, pool)
        setattr(bad, field, value)
        assert code_of(bad) == code, field
    assert code_of(good, -1) == 1  # negative count without a device-side one
    torch.cuda.synchronize()
    assert float(out.max()) == -7.0
