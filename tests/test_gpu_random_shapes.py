"""Seeded random shapes: the eviction pass and the decode steps against the oracle over a spread of
head counts, lengths around the kernels' tile and chunk sizes, window and budget extremes, both head
modes, both element types, contiguous and paged caches.  Every case is reproducible from its seed."""
import numpy as np
import pytest

import synth
from tests import gpu_util as gu
from tests.test_gpu_parity import decode_case, per_query_case, rand_case, select_parity
from tests.test_gpu_paged import paged_case

pytestmark = pytest.mark.gpu
BF16, F32 = synth.BF16, synth.F32

# lengths that straddle the 64-token block, the 1024-token score chunk and the 4096-token combine chunk
EDGE_L = [65, 127, 128, 129, 1023, 1024, 1025, 2049, 4095, 4096, 4097, 8191, 12289]


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = BF16 if rng.random() < 0.7 else F32
    d = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
    Hkv = int(rng.choice([1, 2, 3]))
    P = int(rng.choice([1, 2]))
    if rng.random() < 0.5:
        L = int(rng.choice(EDGE_L))
    else:
        L = int(rng.integers(70, 30000))
    S = int(rng.choice([0, 1, 4, 17, 64, 100]))
    S = min(S, L // 4)
    W = int(rng.choice([1, 2, 16, 63, 64, 65, 300]))
    W = max(1, min(W, L // 3))
    E = L - S - W
    kind = rng.random()
    if kind < 0.1:
        k = 0
    elif kind < 0.2:
        k = E
    elif kind < 0.3:
        k = max(E - 1, 0)
    elif kind < 0.65:
        k = int(rng.integers(1, max(2, E // 12 + 1)))   # small share: the pre-filtered path where it applies
    else:
        k = int(rng.integers(1, E + 1))
    return dtype, P, G * Hkv, Hkv, d, L, S, W, min(k, E)


@pytest.mark.parametrize("seed", range(60))
def test_select_random_shape(ref, seed):
    dtype, P, Hq, Hkv, d, L, S, W, k = draw(seed)
    print(f"seed {seed}: dtype {dtype} P {P} Hq {Hq} Hkv {Hkv} d {d} L {L} S {S} W {W} k {k}", flush=True)
    q, K, V = rand_case(5000 + seed, P, Hq, Hkv, d, L, dtype)
    select_parity(ref, dtype, q, K, V, S, W, k)


@pytest.mark.parametrize("seed", range(60, 80))
def test_select_paged_random_shape(ref, seed):
    dtype, P, Hq, Hkv, d, L, S, W, k = draw(seed)
    rng = np.random.default_rng(seed)
    page = int(rng.choice([16, 32, 64, 256, 2048]))
    print(f"seed {seed}: dtype {dtype} P {P} Hq {Hq} Hkv {Hkv} d {d} L {L} S {S} W {W} k {k} page {page}", flush=True)
    paged_case(ref, dtype, P, Hq, Hkv, d, L, S, W, k, page, token_major=bool(rng.integers(2)),
               want_scores=bool(rng.integers(2)), seed=seed)


@pytest.mark.parametrize("seed", range(80, 100))
def test_per_query_random_shape(ref, seed):
    dtype, P, Hq, Hkv, d, L, S, W, k = draw(seed)
    G = Hq // Hkv
    k = min(k, (L - S - W) // max(G, 1), 600)   # G lists share the candidates; keep the reduced rows short
    print(f"seed {seed}: dtype {dtype} P {P} Hq {Hq} Hkv {Hkv} d {d} L {L} S {S} W {W} k {k}", flush=True)
    per_query_case(ref, dtype, P, Hq, Hkv, d, L, S, W, k, 2, seed=7000 + seed)


@pytest.mark.parametrize("seed", range(100, 140))
def test_decode_random_shape(ref, seed):
    rng = np.random.default_rng(seed)
    dtype = BF16 if rng.random() < 0.75 else F32
    d = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 4, 5, 7, 8, 11, 16, 20]))
    Hkv = int(rng.choice([1, 2, 4]))
    rows = int(rng.choice([1, 3, 8, 40, 192, 260]))
    P = max(1, rows // Hkv)
    S = int(rng.choice([0, 3, 4, 33, 128]))
    k = int(rng.choice([0, 1, 31, 95, 200, 700]))
    W = int(rng.choice([1, 2, 15, 32, 100]))
    if P * Hkv >= 40:
        k = min(k, 200)
    steps = int(rng.integers(1, 5))
    print(f"seed {seed}: dtype {dtype} P {P} Hq {G * Hkv} Hkv {Hkv} d {d} S {S} k {k} W {W} steps {steps}", flush=True)
    decode_case(ref, dtype, P, G * Hkv, Hkv, d, S, k, W, steps, seed=9000 + seed, grow=bool(rng.random() < 0.25))
