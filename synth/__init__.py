"""Seeded synthetic KV caches shaped like the paper's models (Sec. 3.1: Llama-3.1-8B,
Llama-3-8B-ProLong-512k, Qwen2.5-7B) for the eviction pass and decode attention.

This module is the only code that the CPU oracle's tests and the HIP path's tests
share.  It holds no arithmetic of the method itself: it produces inputs.

Recipe
------
* Base values of every tensor are i.i.d. N(0,1): an integer counter hash
  (`counter_rng.h`) picks one of 65,536 entries of an inverse-normal-CDF table
  (built here in fp64 with scipy, then rounded to the tensor's element type).
  The same hash runs on the host (`fill_host.c`) and on the GPU
  (`fill_device.hip`), bit for bit.
* Needles: per (problem, KV head) a few distinct positions among the eviction
  candidates get K = a * unit(q_last of one query head of the group) + 0.1 * z,
  z ~ N(0, I), so that a handful of tokens carry most of the attention mass
  (the sparsity the paper's Sec. 1 describes).  Needle rows are computed here on
  the host in fp64, rounded once, and written over the base fill by both sides.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from functools import lru_cache

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_MASK = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15

# tensor ids of the independent streams
T_QLAST, T_K, T_V, T_QSTEP, T_KNEW, T_VNEW, T_NEEDLE_POS, T_NEEDLE_Z, T_NEEDLE_A = range(1, 10)

BF16, F32 = 0, 1


# ----------------------------------------------------------------------------- configs
@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    seed: int
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    L: int
    n_sink: int
    n_recent: int
    k: int
    n_needles: int
    needle_scale: tuple  # (lo, hi); lo == hi means constant
    needle_log_uniform: bool
    decode_steps: int

    @property
    def n_problems(self) -> int:
        return self.n_layers * self.batch

    @property
    def G(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def rows(self) -> int:
        return self.n_problems * self.n_kv_heads

    @property
    def E(self) -> int:
        return self.L - self.n_sink - self.n_recent

    @property
    def budget(self) -> int:
        return self.n_sink + self.k + self.n_recent

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == BF16 else 4

    def with_(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    "C1": Config("C1", 0x5A6E0001, 1, 1, 4, 2, 64, F32, 4096, 4, 64, 188, 16, (3.0, 3.0), False, 8),
    "C2": Config("C2", 0x5A6E0002, 32, 1, 32, 8, 128, BF16, 32768, 4, 256, 1788, 64, (3.0, 3.0), False, 128),
    "C3": Config("C3", 0x5A6E0003, 32, 1, 32, 8, 128, BF16, 131072, 4, 512, 3580, 256, (2.0, 4.0), False, 256),
    "C4": Config("C4", 0x5A6E0004, 28, 4, 28, 4, 128, BF16, 131072, 4, 128, 892, 128, (3.0, 3.0), False, 256),
    "C5": Config("C5", 0x5A6E0005, 32, 1, 32, 8, 128, BF16, 524288, 4, 1024, 7164, 512, (3.0, 3.0), True, 512),
}


# ----------------------------------------------------------------------------- hash (numpy mirror of counter_rng.h)
def _mix64(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _mix64_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, tensor_id: int) -> int:
    return _mix64_int(_mix64_int(seed + _GOLDEN) + tensor_id * _GOLDEN)


def bits64(key: int, ctr: np.ndarray) -> np.ndarray:
    ctr = np.asarray(ctr, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(np.uint64(key) + (ctr + np.uint64(1)) * np.uint64(_GOLDEN))


def u16(key: int, elem: np.ndarray) -> np.ndarray:
    elem = np.asarray(elem, dtype=np.uint64)
    h = bits64(key, elem >> np.uint64(2))
    return ((h >> (np.uint64(16) * (elem & np.uint64(3)))) & np.uint64(0xFFFF)).astype(np.int64)


# ----------------------------------------------------------------------------- tables and rounding
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))
    return (b >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


@lru_cache(maxsize=None)
def normal_table64() -> np.ndarray:
    from scipy.special import ndtri

    t = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    t.setflags(write=False)
    return t


@lru_cache(maxsize=None)
def normal_table(dtype: int) -> np.ndarray:
    """The lookup table in the tensor's element type (uint16 bf16 bits or float32)."""
    t32 = normal_table64().astype(np.float32)
    t = f32_to_bf16_bits(t32) if dtype == BF16 else t32
    t.setflags(write=False)
    return t


def round_to_dtype(x64: np.ndarray, dtype: int) -> np.ndarray:
    x32 = np.asarray(x64, dtype=np.float64).astype(np.float32)
    return f32_to_bf16_bits(x32) if dtype == BF16 else x32


def to_f64(x: np.ndarray, dtype: int) -> np.ndarray:
    return bf16_bits_to_f64(x) if dtype == BF16 else np.asarray(x, dtype=np.float32).astype(np.float64)


def np_dtype(dtype: int):
    return np.uint16 if dtype == BF16 else np.float32


# ----------------------------------------------------------------------------- native fills
def _build(src: str, out: str, cmd: list) -> None:
    srcs = [os.path.join(_HERE, src), os.path.join(_HERE, "counter_rng.h")]
    if os.path.exists(out) and all(os.path.getmtime(out) >= os.path.getmtime(s) for s in srcs):
        return
    subprocess.check_call(cmd + [os.path.join(_HERE, src), "-o", out], cwd=_HERE)


def build_host(force: bool = False) -> str:
    out = os.path.join(_HERE, "libsagekv_synth_host.so")
    if force and os.path.exists(out):
        os.remove(out)
    _build("fill_host.c", out, ["gcc", "-O2", "-shared", "-fPIC", "-std=c99"])
    return out


def build_device(force: bool = False) -> str:
    out = os.path.join(_HERE, "libsagekv_synth_hip.so")
    if force and os.path.exists(out):
        os.remove(out)
    _build(
        "fill_device.hip",
        out,
        ["hipcc", "--offload-arch=gfx950", "-O3", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"],
    )
    return out


@lru_cache(maxsize=None)
def _host_lib():
    lib = ctypes.CDLL(build_host())
    lib.synth_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64,
                                    ctypes.c_uint64, ctypes.c_uint64]
    lib.synth_fill_host.restype = ctypes.c_int
    lib.synth_stream_key_c.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
    lib.synth_stream_key_c.restype = ctypes.c_uint64
    lib.synth_bits64_c.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
    lib.synth_bits64_c.restype = ctypes.c_uint64
    return lib


@lru_cache(maxsize=None)
def _device_lib():
    path = os.path.join(_HERE, "libsagekv_synth_hip.so")
    if not os.path.exists(path):
        path = build_device()
    lib = ctypes.CDLL(path)
    lib.synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]
    lib.synth_fill_device.restype = ctypes.c_int
    return lib


def fill_host(key: int, first_elem: int, n: int, dtype: int) -> np.ndarray:
    """n consecutive logical elements of a stream, in the element type's bits."""
    out = np.empty(n, dtype=np_dtype(dtype))
    tab = normal_table(dtype)
    rc = _host_lib().synth_fill_host(out.ctypes.data, out.itemsize, tab.ctypes.data, key, first_elem, n)
    if rc != 0:
        raise RuntimeError(f"synth_fill_host failed: {rc}")
    return out


_dev_tables = {}


def fill_device(t, key: int, first_elem: int = 0) -> None:
    """Fill a contiguous torch device tensor (bf16 or fp32) with the stream's elements
    [first_elem, first_elem + t.numel())."""
    import torch

    assert t.is_cuda and t.is_contiguous()
    dtype = BF16 if t.dtype == torch.bfloat16 else F32
    assert t.dtype in (torch.bfloat16, torch.float32)
    dk = (t.device.index, dtype)
    if dk not in _dev_tables:
        tab = normal_table(dtype)
        tt = torch.from_numpy(tab.view(np.int16).copy() if dtype == BF16 else tab.copy()).to(t.device)
        _dev_tables[dk] = tt
    tab = _dev_tables[dk]
    stream = torch.cuda.current_stream(t.device).cuda_stream
    rc = _device_lib().synth_fill_device(t.data_ptr(), t.element_size(), tab.data_ptr(), key, first_elem,
                                         t.numel(), stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_device failed: {rc}")


# ----------------------------------------------------------------------------- tensors of a config
def q_last_host(cfg: Config) -> np.ndarray:
    """[n_problems, Hq, d] in the config's element type."""
    n = cfg.n_problems * cfg.n_q_heads * cfg.head_dim
    return fill_host(stream_key(cfg.seed, T_QLAST), 0, n, cfg.dtype).reshape(cfg.n_problems, cfg.n_q_heads, cfg.head_dim)


def needles(cfg: Config, q_last: np.ndarray | None = None):
    """Needle positions [rows, n_needles] (int64, distinct per row, inside the candidate range)
    and the K rows to write there [rows, n_needles, d] in the config's element type."""
    if q_last is None:
        q_last = q_last_host(cfg)
    rows, nn, d, G = cfg.rows, cfg.n_needles, cfg.head_dim, cfg.G
    S, E = cfg.n_sink, cfg.E
    kpos = stream_key(cfg.seed, T_NEEDLE_POS)
    pos = np.empty((rows, nn), dtype=np.int64)
    for r in range(rows):
        taken = set()
        for n in range(nn):
            attempt = 0
            while True:
                ctr = ((r * nn + n) << 8) + attempt
                h = int(bits64(kpos, np.uint64(ctr)))
                if cfg.needle_log_uniform:
                    u = (h >> 11) / float(1 << 53)
                    p = S + max(int(np.floor(float(E) ** u)) - 1, 0)
                else:
                    p = S + h % E
                if p not in taken or attempt >= 255:
                    break
                attempt += 1
            if p in taken:  # 256 collisions in a row: take the first free slot
                p = next(x for x in range(S, S + E) if x not in taken)
            taken.add(p)
            pos[r, n] = p
    # scale a
    lo, hi = cfg.needle_scale
    ka = stream_key(cfg.seed, T_NEEDLE_A)
    ua = (bits64(ka, np.arange(rows * nn, dtype=np.uint64)) >> np.uint64(11)).astype(np.float64) / float(1 << 53)
    a = (lo + (hi - lo) * ua).reshape(rows, nn)
    # noise z from the fp64 table
    kz = stream_key(cfg.seed, T_NEEDLE_Z)
    z = normal_table64()[u16(kz, np.arange(rows * nn * d, dtype=np.uint64))].reshape(rows, nn, d)
    # target query head of the group: g = n mod G
    q64 = to_f64(q_last, cfg.dtype).reshape(cfg.n_problems, cfg.n_kv_heads, G, d).reshape(rows, G, d)
    qhat = q64 / np.linalg.norm(q64, axis=-1, keepdims=True)
    g = np.arange(nn) % G
    vals = a[:, :, None] * qhat[:, g, :] + 0.1 * z
    return pos, round_to_dtype(vals, cfg.dtype)


def kv_row_host(cfg: Config, which: str, row: int, needle_pos=None, needle_rows=None) -> np.ndarray:
    """One (problem, KV head) row of K or V, [L, d], needles applied to K."""
    n = cfg.L * cfg.head_dim
    key = stream_key(cfg.seed, T_K if which == "K" else T_V)
    x = fill_host(key, row * n, n, cfg.dtype).reshape(cfg.L, cfg.head_dim)
    if which == "K" and needle_pos is not None:
        x[needle_pos[row]] = needle_rows[row]
    return x


def kv_host(cfg: Config):
    """Whole K and V of a (small) config on the host: [n_problems, Hkv, L, d] each."""
    q = q_last_host(cfg)
    pos, nrows = needles(cfg, q)
    K = np.stack([kv_row_host(cfg, "K", r, pos, nrows) for r in range(cfg.rows)])
    V = np.stack([kv_row_host(cfg, "V", r) for r in range(cfg.rows)])
    shp = (cfg.n_problems, cfg.n_kv_heads, cfg.L, cfg.head_dim)
    return q, K.reshape(shp), V.reshape(shp), pos


def decode_inputs_host(cfg: Config, step: int):
    """(q [P,Hq,d], k_new [P,Hkv,d], v_new [P,Hkv,d]) of decode step `step`."""
    P, d = cfg.n_problems, cfg.head_dim
    nq, nk = P * cfg.n_q_heads * d, P * cfg.n_kv_heads * d
    q = fill_host(stream_key(cfg.seed, T_QSTEP), step * nq, nq, cfg.dtype).reshape(P, cfg.n_q_heads, d)
    kn = fill_host(stream_key(cfg.seed, T_KNEW), step * nk, nk, cfg.dtype).reshape(P, cfg.n_kv_heads, d)
    vn = fill_host(stream_key(cfg.seed, T_VNEW), step * nk, nk, cfg.dtype).reshape(P, cfg.n_kv_heads, d)
    return q, kn, vn


# ----------------------------------------------------------------------------- device side
def torch_dtype(dtype: int):
    import torch

    return torch.bfloat16 if dtype == BF16 else torch.float32


def host_to_torch(x: np.ndarray, dtype: int, device="cuda"):
    import torch

    if dtype == BF16:
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)


def torch_to_host(t, dtype: int) -> np.ndarray:
    import torch

    t = t.detach().cpu().contiguous()
    if dtype == BF16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def kv_device(cfg: Config, device="cuda"):
    """q_last, K, V on the device, generated there (needle rows uploaded), plus needle positions."""
    import torch

    td = torch_dtype(cfg.dtype)
    shp = (cfg.n_problems, cfg.n_kv_heads, cfg.L, cfg.head_dim)
    K = torch.empty(shp, dtype=td, device=device)
    V = torch.empty(shp, dtype=td, device=device)
    fill_device(K, stream_key(cfg.seed, T_K))
    fill_device(V, stream_key(cfg.seed, T_V))
    qh = q_last_host(cfg)
    pos, nrows = needles(cfg, qh)
    Kr = K.view(cfg.rows, cfg.L, cfg.head_dim)
    r_idx = torch.arange(cfg.rows, device=device).repeat_interleave(cfg.n_needles)
    p_idx = torch.from_numpy(pos.reshape(-1)).to(device)
    Kr[r_idx, p_idx] = host_to_torch(nrows.reshape(-1, cfg.head_dim), cfg.dtype, device)
    q = host_to_torch(qh, cfg.dtype, device)
    torch.cuda.synchronize()
    return q, K, V, pos


def decode_inputs_device(cfg: Config, step: int, device="cuda"):
    q, kn, vn = decode_inputs_host(cfg, step)
    return tuple(host_to_torch(x, cfg.dtype, device) for x in (q, kn, vn))
