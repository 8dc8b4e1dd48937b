"""The seeded input generator: host C fill, numpy mirror and table agree; needles are well formed."""
import numpy as np

import synth


def test_numpy_hash_matches_c():
    lib = synth._host_lib()
    key = synth.stream_key(123, 4)
    assert key == lib.synth_stream_key_c(123, 4)
    ctr = np.array([0, 1, 2, 12345678901234, 2**63 + 5], dtype=np.uint64)
    got = synth.bits64(key, ctr)
    for c, g in zip(ctr.tolist(), got.tolist()):
        assert g == lib.synth_bits64_c(key, c)


def test_fill_matches_table_lookup_and_is_offset_consistent():
    key = synth.stream_key(9, synth.T_K)
    for dtype in (synth.BF16, synth.F32):
        a = synth.fill_host(key, 0, 1000, dtype)
        idx = synth.u16(key, np.arange(1000, dtype=np.uint64))
        np.testing.assert_array_equal(a, synth.normal_table(dtype)[idx])
        b = synth.fill_host(key, 333, 100, dtype)
        np.testing.assert_array_equal(b, a[333:433])


def test_values_look_standard_normal():
    x = synth.to_f64(synth.fill_host(synth.stream_key(1, 2), 0, 400_000, synth.BF16), synth.BF16)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs(np.mean(x > 1.0) - 0.1587) < 0.005


def test_needles_distinct_in_range_and_aligned_with_query():
    cfg = synth.CONFIGS["C1"]
    q = synth.q_last_host(cfg)
    pos, rows = synth.needles(cfg, q)
    assert pos.shape == (cfg.rows, cfg.n_needles)
    for r in range(cfg.rows):
        assert len(set(pos[r].tolist())) == cfg.n_needles
        assert pos[r].min() >= cfg.n_sink and pos[r].max() < cfg.L - cfg.n_recent
    q64 = synth.to_f64(q, cfg.dtype).reshape(cfg.rows, cfg.G, cfg.head_dim)
    r64 = synth.to_f64(rows, cfg.dtype)
    for n in range(cfg.n_needles):
        g = n % cfg.G
        logit = (r64[:, n] * q64[:, g]).sum(-1) / np.sqrt(cfg.head_dim)
        assert np.all(logit > 2.0)  # a * |q| / sqrt(d) ~ 3


def test_log_uniform_needles():
    cfg = synth.CONFIGS["C5"].with_(n_layers=1, n_kv_heads=1, n_q_heads=4, L=65536, n_needles=64)
    pos, _ = synth.needles(cfg)
    assert np.median(pos) < cfg.L / 8  # log-uniform piles up near the start
    assert len(set(pos[0].tolist())) == 64
