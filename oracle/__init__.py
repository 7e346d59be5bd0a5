"""ctypes loader for the CPU oracle (oracle/fss_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, by __graft_entry__.smoke() and by the
CPU-baseline leg of bench.py.  The product package never imports this module.

`build()` compiles the C file with gcc; `lib()` loads the shared object (building it on
first use when no built copy is present).  The wrappers below only marshal numpy arrays;
all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fss_oracle.c")
_SO = os.path.join(_HERE, "libfss_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared", _SRC, "-o", _SO]
        subprocess.run(cmd, check=True)
    return _SO


def load(path: str) -> C.CDLL:
    """Load an oracle shared object and declare its argument types."""
    L = C.CDLL(path)
    u8p, u32p, i32p, vp = (C.POINTER(C.c_uint8), C.POINTER(C.c_uint32), C.POINTER(C.c_int32), C.c_void_p)
    L.oracle_init.restype = None
    L.oracle_aes128_encrypt.argtypes = [u8p, u8p, u8p]
    L.oracle_aes128_encrypt.restype = None
    L.oracle_prg.argtypes = [C.c_int, u8p, u8p]
    L.oracle_prg.restype = None
    L.oracle_prg_key.argtypes = [C.c_int, u8p]
    L.oracle_prg_key.restype = None
    for name in ("oracle_cmp_key_bytes", "oracle_eq_key_bytes"):
        f = getattr(L, name)
        f.argtypes = [C.c_int, C.c_size_t]
        f.restype = C.c_size_t
    for name in ("oracle_cmp_key_bits_logical", "oracle_eq_key_bits_logical"):
        f = getattr(L, name)
        f.argtypes = [C.c_int]
        f.restype = C.c_size_t
    for name in ("oracle_cmp_gen", "oracle_eq_gen"):
        f = getattr(L, name)
        f.argtypes = [C.c_int, C.c_size_t, u32p, u32p, u8p, u8p, vp, vp]
        f.restype = C.c_int
    for name in ("oracle_cmp_eval", "oracle_eq_eval"):
        f = getattr(L, name)
        f.argtypes = [C.c_int, C.c_int, C.c_size_t, vp, u32p, u32p]
        f.restype = C.c_int
    for name in ("oracle_cmp_eval_all_x", "oracle_eq_eval_all_x"):
        f = getattr(L, name)
        f.argtypes = [C.c_int, C.c_int, C.c_size_t, vp, C.c_size_t, u32p]
        f.restype = C.c_int
    L.oracle_eval_trace.argtypes = [C.c_int, C.c_int, C.c_int, C.c_size_t, vp, C.c_size_t, C.c_uint32,
                                    u8p, i32p, u32p, i32p, u32p, u32p]
    L.oracle_eval_trace.restype = C.c_int
    L.oracle_sign_mask.argtypes = [C.c_int, C.c_size_t, vp, u32p, u32p]
    L.oracle_sign_mask.restype = C.c_int
    L.oracle_sign_eval.argtypes = [C.c_int, C.c_int, C.c_size_t, vp, u32p, u32p, u32p]
    L.oracle_sign_eval.restype = C.c_int
    L.oracle_relu_open.argtypes = [C.c_int, C.c_int, C.c_size_t, vp, u32p, u32p, u32p, u32p, u32p, u32p, u32p]
    L.oracle_relu_open.restype = C.c_int
    L.oracle_relu_finish.argtypes = [C.c_int, C.c_int, C.c_size_t, u32p, u32p, u32p, u32p, u32p, u32p, u32p, u32p]
    L.oracle_relu_finish.restype = C.c_int
    L.oracle_eq_mask.argtypes = [C.c_int, C.c_size_t, vp, u32p, u32p]
    L.oracle_eq_masked_eval.argtypes = [C.c_int, C.c_int, C.c_size_t, vp, u32p, u32p, u32p]
    L.oracle_argmax_diff_mask.argtypes = [C.c_int, C.c_size_t, C.c_int, vp, u32p, u32p]
    L.oracle_argmax_count_mask.argtypes = [C.c_int, C.c_int, C.c_size_t, C.c_int, u32p, vp, u32p]
    L.oracle_maxpool_unroll.argtypes = [C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_int, u32p, u32p]
    L.oracle_mul_open.argtypes = [C.c_int, C.c_size_t, u32p, u32p, u32p, u32p, u32p, u32p]
    L.oracle_dot_finish.argtypes = [C.c_int, C.c_int, C.c_size_t, C.c_int, u32p, u32p, u32p, u32p, u32p, u32p, u32p, u32p]
    for _name in ("oracle_eq_mask", "oracle_eq_masked_eval", "oracle_argmax_diff_mask", "oracle_argmax_count_mask",
                  "oracle_maxpool_unroll", "oracle_mul_open", "oracle_dot_finish"):
        getattr(L, _name).restype = C.c_int
    L.oracle_set_threads.argtypes = [C.c_int]
    L.oracle_set_threads.restype = C.c_int
    L.oracle_init()
    return L


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = load(_SO)
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _u32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint32)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def aes128_encrypt(key: bytes, block: bytes) -> bytes:
    k = np.frombuffer(bytes(key), dtype=np.uint8).copy()
    b = np.frombuffer(bytes(block), dtype=np.uint8).copy()
    o = np.zeros(16, dtype=np.uint8)
    lib().oracle_aes128_encrypt(_p(k, C.c_uint8), _p(b, C.c_uint8), _p(o, C.c_uint8))
    return o.tobytes()


def prg(m: int, block: bytes) -> bytes:
    b = np.frombuffer(bytes(block), dtype=np.uint8).copy()
    o = np.zeros(16, dtype=np.uint8)
    lib().oracle_prg(m, _p(b, C.c_uint8), _p(o, C.c_uint8))
    return o.tobytes()


def prg_key(m: int) -> bytes:
    o = np.zeros(16, dtype=np.uint8)
    lib().oracle_prg_key(m, _p(o, C.c_uint8))
    return o.tobytes()


def key_bytes(kind: str, n: int, batch: int) -> int:
    f = lib().oracle_cmp_key_bytes if kind == "cmp" else lib().oracle_eq_key_bytes
    return int(f(n, batch))


def key_bits_logical(kind: str, n: int) -> int:
    f = lib().oracle_cmp_key_bits_logical if kind == "cmp" else lib().oracle_eq_key_bits_logical
    return int(f(n))


def gen(kind: str, n: int, alpha, r, seed0, seed1) -> Tuple[np.ndarray, np.ndarray]:
    """Both parties' key buffers (uint8 arrays) for a batch of KeyGen arguments."""
    alpha, r, seed0, seed1 = _u32(alpha), _u32(r), _u8(seed0), _u8(seed1)
    batch = alpha.shape[0]
    assert r.shape == (batch,) and seed0.shape == (batch, 16) and seed1.shape == (batch, 16)
    nbytes = key_bytes(kind, n, batch)
    if nbytes == 0 and batch > 0:
        raise ValueError("bad n")
    k0 = np.zeros(max(nbytes, 1), dtype=np.uint8)[:nbytes]
    k1 = np.zeros(max(nbytes, 1), dtype=np.uint8)[:nbytes]
    f = lib().oracle_cmp_gen if kind == "cmp" else lib().oracle_eq_gen
    rc = f(n, batch, _p(alpha, C.c_uint32), _p(r, C.c_uint32), _p(seed0, C.c_uint8), _p(seed1, C.c_uint8),
           k0.ctypes.data, k1.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle gen failed: {rc}")
    return k0, k1


def eval_(kind: str, party: int, n: int, key: np.ndarray, x) -> np.ndarray:
    x = _u32(x)
    batch = x.shape[0]
    out = np.zeros(batch, dtype=np.uint32)
    f = lib().oracle_cmp_eval if kind == "cmp" else lib().oracle_eq_eval
    rc = f(party, n, batch, key.ctypes.data, _p(x, C.c_uint32), _p(out, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle eval failed: {rc}")
    return out


def eval_all_x(kind: str, party: int, n: int, batch: int, key: np.ndarray, e: int) -> np.ndarray:
    out = np.zeros(1 << n, dtype=np.uint32)
    f = lib().oracle_cmp_eval_all_x if kind == "cmp" else lib().oracle_eq_eval_all_x
    rc = f(party, n, batch, key.ctypes.data, e, _p(out, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle eval_all_x failed: {rc}")
    return out


def eval_trace(kind: str, party: int, n: int, batch: int, key: np.ndarray, e: int, x: int) -> dict:
    s = np.zeros((n + 1, 16), dtype=np.uint8)
    t = np.zeros(n + 1, dtype=np.int32)
    sigma = np.zeros(n + 1, dtype=np.uint32)
    tau = np.zeros(n + 1, dtype=np.int32)
    outs = np.zeros(n + 2, dtype=np.uint32)
    share = C.c_uint32(0)
    rc = lib().oracle_eval_trace(1 if kind == "cmp" else 0, party, n, batch, key.ctypes.data, e, int(x),
                                 _p(s, C.c_uint8), _p(t, C.c_int32), _p(sigma, C.c_uint32), _p(tau, C.c_int32),
                                 _p(outs, C.c_uint32), C.byref(share))
    if rc != 0:
        raise ValueError(f"oracle trace failed: {rc}")
    return {"s": s, "t": t, "sigma": sigma, "tau": tau, "out": outs, "share": int(share.value)}


def sign_mask(n: int, key: np.ndarray, y_share) -> np.ndarray:
    y_share = _u32(y_share)
    out = np.zeros(y_share.shape[0], dtype=np.uint32)
    rc = lib().oracle_sign_mask(n, y_share.shape[0], key.ctypes.data, _p(y_share, C.c_uint32), _p(out, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle sign_mask failed: {rc}")
    return out


def sign_eval(party: int, n: int, key: np.ndarray, masked0, masked1) -> np.ndarray:
    m0, m1 = _u32(masked0), _u32(masked1)
    out = np.zeros(m0.shape[0], dtype=np.uint32)
    rc = lib().oracle_sign_eval(party, n, m0.shape[0], key.ctypes.data, _p(m0, C.c_uint32), _p(m1, C.c_uint32), _p(out, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle sign_eval failed: {rc}")
    return out


def relu_open(party: int, n: int, key: np.ndarray, masked0, masked1, y_share, tri_a, tri_b):
    arrs = [_u32(a) for a in (masked0, masked1, y_share, tri_a, tri_b)]
    batch = arrs[0].shape[0]
    delta = np.zeros(batch, dtype=np.uint32)
    eps = np.zeros(batch, dtype=np.uint32)
    rc = lib().oracle_relu_open(party, n, batch, key.ctypes.data, *[_p(a, C.c_uint32) for a in arrs],
                                _p(delta, C.c_uint32), _p(eps, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle relu_open failed: {rc}")
    return delta, eps


def relu_finish(party: int, n: int, delta0, delta1, eps0, eps1, tri_a, tri_b, tri_c) -> np.ndarray:
    arrs = [_u32(a) for a in (delta0, delta1, eps0, eps1, tri_a, tri_b, tri_c)]
    batch = arrs[0].shape[0]
    out = np.zeros(batch, dtype=np.uint32)
    rc = lib().oracle_relu_finish(party, n, batch, *[_p(a, C.c_uint32) for a in arrs], _p(out, C.c_uint32))
    if rc != 0:
        raise ValueError(f"oracle relu_finish failed: {rc}")
    return out


def _call(name, *args):
    rc = getattr(lib(), name)(*args)
    if rc != 0:
        raise ValueError(f"{name} failed: {rc}")


def eq_mask(n: int, key: np.ndarray, y_share) -> np.ndarray:
    y_share = _u32(y_share)
    out = np.zeros(y_share.shape[0], dtype=np.uint32)
    _call("oracle_eq_mask", n, y_share.shape[0], key.ctypes.data, _p(y_share, C.c_uint32), _p(out, C.c_uint32))
    return out


def eq_masked_eval(party: int, n: int, key: np.ndarray, masked0, masked1) -> np.ndarray:
    m0, m1 = _u32(masked0), _u32(masked1)
    out = np.zeros(m0.shape[0], dtype=np.uint32)
    _call("oracle_eq_masked_eval", party, n, m0.shape[0], key.ctypes.data, _p(m0, C.c_uint32), _p(m1, C.c_uint32), _p(out, C.c_uint32))
    return out


def argmax_diff_mask(n: int, rows: int, m: int, cmp_key: np.ndarray, x_share) -> np.ndarray:
    x_share = _u32(x_share).reshape(rows, m)
    out = np.zeros(rows * m * (m - 1), dtype=np.uint32)
    _call("oracle_argmax_diff_mask", n, rows, m, cmp_key.ctypes.data, _p(x_share, C.c_uint32), _p(out, C.c_uint32))
    return out


def argmax_count_mask(party: int, n: int, rows: int, m: int, w_share, eq_key: np.ndarray) -> np.ndarray:
    w_share = _u32(w_share)
    out = np.zeros(rows * m, dtype=np.uint32)
    _call("oracle_argmax_count_mask", party, n, rows, m, _p(w_share, C.c_uint32), eq_key.ctypes.data, _p(out, C.c_uint32))
    return out


def maxpool_unroll(channels: int, h: int, w: int, k: int, s: int, x_share) -> np.ndarray:
    x_share = _u32(x_share).reshape(channels, h, w)
    oh, ow = (h - k) // s + 1, (w - k) // s + 1
    out = np.zeros((channels * oh * ow, k * k), dtype=np.uint32)
    _call("oracle_maxpool_unroll", channels, h, w, k, s, _p(x_share, C.c_uint32), _p(out, C.c_uint32))
    return out


def mul_open(n: int, u_share, v_share, tri_a, tri_b):
    arrs = [_u32(a).reshape(-1) for a in (u_share, v_share, tri_a, tri_b)]
    delta = np.zeros(arrs[0].shape[0], dtype=np.uint32)
    eps = np.zeros_like(delta)
    _call("oracle_mul_open", n, arrs[0].shape[0], *[_p(a, C.c_uint32) for a in arrs], _p(delta, C.c_uint32), _p(eps, C.c_uint32))
    return delta, eps


def dot_finish(party: int, n: int, rows: int, m: int, delta0, delta1, eps0, eps1, tri_a, tri_b, tri_c) -> np.ndarray:
    arrs = [_u32(a).reshape(-1) for a in (delta0, delta1, eps0, eps1, tri_a, tri_b, tri_c)]
    out = np.zeros(rows, dtype=np.uint32)
    _call("oracle_dot_finish", party, n, rows, m, *[_p(a, C.c_uint32) for a in arrs], _p(out, C.c_uint32))
    return out


def set_threads(threads: int) -> int:
    return int(lib().oracle_set_threads(threads))


def split_key(kind: str, n: int, batch: int, key: np.ndarray) -> dict:
    """Views of the planes of a key buffer (layout documented at the top of fss_oracle.c)."""
    bp = (batch + 63) // 64 * 64
    off = 0

    def take(nbytes, dtype, shape):
        nonlocal off
        v = key[off:off + nbytes].view(dtype).reshape(shape)
        off += nbytes
        return v

    d = {"bp": bp}
    d["alpha_share"] = take(4 * bp, np.uint32, (bp,))
    d["seed"] = take(16 * bp, np.uint8, (bp, 16))
    cw = 4 if kind == "cmp" else 2
    d["ctrl"] = take(4 * cw * bp, np.uint32, (bp, cw))
    d["s_cw"] = take(16 * n * bp, np.uint8, (n, bp, 16))
    if kind == "cmp":
        d["sigma_cw"] = take(4 * n * bp, np.uint32, (n, bp))
        d["leaf"] = take(4 * n * bp, np.uint32, (n, bp))
    d["last"] = take(4 * bp, np.uint32, (bp,))
    assert off == key.shape[0]
    return d
