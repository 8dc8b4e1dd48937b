"""Eviction pass over a paged cache (block table + page pools).  The layout only says where a
token lives, so the oracle runs on the logical cache and the paged HIP path must give the same
kept sets, reduced K/V and scores.  Unused pool pages and the unused tail of a problem's last page
hold NaN patterns: a read outside the logical cache would poison the result."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu
from tests.test_gpu_parity import rand_case

pytestmark = pytest.mark.gpu
BF16, F32 = synth.BF16, synth.F32


def to_pages(X, page_size, table, n_pages, token_major, dtype):
    """Logical [P,Hkv,L,d] -> pool [n_pages,Hkv,page,d] (or [n_pages,page,Hkv,d] when token_major)."""
    P, Hkv, L, d = X.shape
    nan = np.uint16(0x7FC1) if dtype == BF16 else np.float32(np.nan)
    pool = np.full((n_pages, Hkv, page_size, d), nan, dtype=X.dtype)
    for p in range(P):
        for j in range(table.shape[1]):
            t0, t1 = j * page_size, min((j + 1) * page_size, L)
            if t0 < L:
                pool[table[p, j], :, : t1 - t0] = X[p, :, t0:t1]
    return np.ascontiguousarray(pool.transpose(0, 2, 1, 3)) if token_major else pool


def paged_case(ref, dtype, P, Hq, Hkv, d, L, S, W, k, page_size, token_major=False, head_mode=0, want_scores=False,
               flags=0, seed=0, q_scale=1.0):
    import torch

    import paper_2503_08879_amd as sk

    q, K, V = rand_case(900 + seed, P, Hq, Hkv, d, L, dtype)
    if q_scale != 1.0:  # peaked attention: a few tokens hold each head's softmax
        q = synth.round_to_dtype(q_scale * synth.to_f64(q, dtype), dtype)
    G = Hq // Hkv
    lists = G if head_mode == 1 else 1
    per = -(-L // page_size)
    n_pages = P * per + 5
    rng = np.random.default_rng(seed)
    table = rng.permutation(n_pages)[: P * per].astype(np.int32).reshape(P, per)
    Kp = synth.host_to_torch(to_pages(K, page_size, table, n_pages, token_major, dtype), dtype)
    Vp = synth.host_to_torch(to_pages(V, page_size, table, n_pages, token_major, dtype), dtype)
    if token_major:
        Kp, Vp = Kp.permute(0, 2, 1, 3), Vp.permute(0, 2, 1, 3)  # logical [n_pages, Hkv, page, d], strided
    qd = synth.host_to_torch(q, dtype)
    tab = torch.from_numpy(table).cuda()
    Bt = S + lists * k + W
    desc, pages = sk.paged_select_desc(qd, Kp, Vp, tab, L, S, W, k, Bt, head_mode=head_mode, flags=flags)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=qd.dtype, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.full((P, Hkv, Bt), -1, dtype=torch.int32, device="cuda")
    scores = torch.empty((P, Hkv * lists, L), dtype=torch.float32, device="cuda") if want_scores else None
    sk.sagekv_select_paged(desc, pages, qd, Kp, Vp, Kc, Vc, kept, scores, ws)
    torch.cuda.synchronize()
    redone = sk.sagekv_select_redone_rows(desc, ws)

    Kc_r, Vc_r, kept_r, s_r = ref.select(dtype, head_mode, q, K, V, S, W, k, want_scores=True)
    got = kept.cpu().numpy()
    n_ex = 0
    for g in range(lists):  # every list against the oracle's, with the near-tie exemption
        cut = lambda a: np.concatenate([a[..., :S], a[..., S + g * k:S + (g + 1) * k], a[..., S + lists * k:]], axis=-1)
        n_ex += gu.check_kept(cut(got), cut(kept_r), s_r[:, :, g], S, W, k)
    if n_ex == 0:
        np.testing.assert_array_equal(synth.torch_to_host(Kc, dtype), Kc_r)
        np.testing.assert_array_equal(synth.torch_to_host(Vc, dtype), Vc_r)
    if want_scores:
        sc = scores.cpu().numpy().reshape(P, Hkv, lists, L)
        gu.check_scores(sc, s_r)
    # and the contiguous layout gives the very same answer
    flat = gu.gpu_select(dtype, q, K, V, S, W, k, want_scores=False, flags=flags, head_mode=head_mode)
    np.testing.assert_array_equal(flat["kept"], got)
    return redone


@pytest.mark.parametrize(
    "page_size,token_major",
    [(16, False), (16, True), (64, False), (256, True), (1024, False), (4096, False)],
)
def test_paged_prefiltered_bf16(ref, page_size, token_major):
    """G = 4, ragged L: pre-filtered path, pages smaller than, equal to and larger than a score chunk."""
    redone = paged_case(ref, BF16, 2, 8, 2, 128, 40000 + 37, 4, 128, 1000, page_size, token_major, seed=page_size)
    assert redone == 0


def test_paged_G7_d64(ref):
    assert paged_case(ref, BF16, 1, 7, 1, 128, 50021, 3, 77, 2000, 32, seed=1) == 0
    assert paged_case(ref, BF16, 2, 4, 2, 64, 33000, 4, 300, 800, 128, token_major=True, seed=2) == 0


def test_paged_dense_with_scores(ref):
    """scores_out forces the dense kernels (MFMA scoring, combine, radix top-k) through the page table."""
    assert paged_case(ref, BF16, 2, 8, 2, 128, 9000, 4, 64, 300, 16, want_scores=True, seed=3) == -1
    assert paged_case(ref, BF16, 1, 4, 1, 64, 5000, 2, 40, 100, 512, token_major=True, want_scores=True, seed=4) == -1


def test_paged_fp32(ref):
    """fp32 caches take the vector-ALU scoring kernel."""
    assert paged_case(ref, F32, 2, 4, 2, 64, 6000, 4, 64, 200, 32, want_scores=True, seed=5) == -1
    assert paged_case(ref, F32, 1, 8, 2, 128, 3000, 0, 16, 50, 16, token_major=True, seed=6) == -1


def test_paged_per_query(ref):
    assert paged_case(ref, BF16, 1, 8, 2, 128, 45000, 64, 128, 256, 64, head_mode=1, seed=7) == 0
    assert paged_case(ref, BF16, 1, 4, 2, 64, 4000, 4, 32, 50, 16, head_mode=1, want_scores=True, seed=8) == -1


def test_paged_short_row_in_one_page(ref):
    """L smaller than a page; k = 0 (sink + window only)."""
    assert paged_case(ref, BF16, 3, 4, 2, 64, 700, 4, 100, 0, 1024, seed=9) == -1


def test_paged_arguments_are_checked():
    import torch

    import paper_2503_08879_amd as sk

    P, Hq, Hkv, d, L, ps = 1, 4, 2, 64, 1000, 64
    q = torch.zeros((P, Hq, d), dtype=torch.bfloat16, device="cuda")
    pool = torch.zeros((20, Hkv, ps, d), dtype=torch.bfloat16, device="cuda")
    tab = torch.zeros((P, 16), dtype=torch.int32, device="cuda")
    desc, pages = sk.paged_select_desc(q, pool, pool, tab, L, 4, 32, 10)
    ws = torch.empty(sk.sagekv_select_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    Kc = torch.zeros((P, Hkv, 46, d), dtype=torch.bfloat16, device="cuda")
    Vc = torch.zeros_like(Kc)
    kept = torch.zeros((P, Hkv, 46), dtype=torch.int32, device="cuda")

    def status(**change):
        pg = sk.PagedKV(pages.block_table, pages.table_pitch, pages.page_size, pages.n_pages, pages.k_stride_page,
                        pages.v_stride_page)
        for name, v in change.items():
            setattr(pg, name, v)
        try:
            sk.sagekv_select_paged(desc, pg, q, pool, pool, Kc, Vc, kept, None, ws)
        except sk.SagekvError as e:
            return e.code
        return 0

    assert status() == 0
    assert status(page_size=8) == 1 and status(page_size=48) == 1     # below 16, not a power of two
    assert status(table_pitch=15) == 1                                 # fewer entries than pages of the row
    assert status(block_table=None) == 1 and status(n_pages=0) == 1
    assert status(k_stride_page=ps * d * Hkv + 4) == 2                 # page not 16-byte aligned
    torch.cuda.synchronize()


@pytest.mark.parametrize("page,want_scores,flags", [(16, False, 0), (64, True, 0), (256, False, 1)])
def test_paged_select_with_peaked_attention(ref, page, want_scores, flags):
    """Queries scaled by 9 over a paged cache: the softmax terms that need an fp64 exponent are recomputed
    from the staged pages (pre-filtered, two-sweep and one-sweep routes)."""
    paged_case(ref, BF16, 1, 4, 2, 128, 70001, 4, 65, 9000, page, want_scores=want_scores, flags=flags, seed=41,
               q_scale=9.0)
