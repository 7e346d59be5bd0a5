"""Thin ctypes binding over the C ABI of include/fss.h -- same names, argument marshalling
only.  Tensors are PyTorch CUDA(HIP) tensors used purely as device buffers; every step of
key generation and evaluation runs inside the HIP kernels of libfss_mi355.so."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_SO = os.path.join(_HERE, "libfss_mi355.so")
_lib: Optional[C.CDLL] = None

EXPORTS = ("fss_cmp_key_bytes", "fss_eq_key_bytes", "fss_cmp_gen", "fss_cmp_eval", "fss_eq_gen", "fss_eq_eval",
           "fss_sign_mask", "fss_sign_eval", "fss_relu_open", "fss_relu_finish", "fss_eq_mask", "fss_eq_masked_eval",
           "fss_argmax_diff_mask", "fss_argmax_count_mask", "fss_maxpool_unroll", "fss_mul_open", "fss_dot_finish",
           "fss_cmp_chunked_key_bytes",
           "fss_cmp_eval_streamed", "fss_cmp_eval_streamed_static", "fss_static_staging_bytes", "fss_prepare", "fss_clock_probe", "fss_wall_clock_khz", "fss_quad_layout_below", "fss_strerror", "fss_last_hip_error")

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


class FssError(RuntimeError):
    def __init__(self, code: int, text: str, hip_error: int = 0):
        super().__init__(f"fss error {code}: {text}" + (f" (hipError_t {hip_error})" if hip_error else ""))
        self.code = code
        self.hip_error = hip_error


def library_path() -> str:
    return _SO


def build(verbose: bool = False) -> str:
    """Compile the HIP sources for gfx950 into libfss_mi355.so (in-tree)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(_CSRC, "fss_kernels.hip"), "-o", _SO]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libfss_mi355.so")
    # the stand-alone micro-benchmark that backs the choice of AES engine
    bench = [hipcc] + [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")] + \
        [os.path.join(_CSRC, "aes_engine_bench.hip"), "-o", os.path.join(_HERE, "aes_engine_bench")]
    res = subprocess.run(bench, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building aes_engine_bench")
    global _lib
    _lib = None
    return _SO


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise FileNotFoundError(
                f"{_SO} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        # PyTorch ships its own copy of the HIP runtime (same soname).  Importing torch first
        # makes the loader bind this library to that copy, so both see the same device
        # context, streams and allocations; loaded the other way round the process would
        # hold two runtimes and every launch here would fail with "no device".
        import torch  # noqa: F401
        L = C.CDLL(_SO)
        vp, sz, i = C.c_void_p, C.c_size_t, C.c_int
        for name in ("fss_cmp_key_bytes", "fss_eq_key_bytes"):
            getattr(L, name).argtypes = [i, sz]
            getattr(L, name).restype = sz
        for name in ("fss_cmp_gen", "fss_eq_gen"):
            getattr(L, name).argtypes = [i, sz, vp, vp, vp, vp, vp, vp, vp]
            getattr(L, name).restype = i
        for name in ("fss_cmp_eval", "fss_eq_eval"):
            getattr(L, name).argtypes = [i, i, sz, vp, vp, vp, vp]
            getattr(L, name).restype = i
        L.fss_sign_mask.argtypes = [i, sz, vp, vp, vp, vp]
        L.fss_sign_eval.argtypes = [i, i, sz, vp, vp, vp, vp, vp]
        L.fss_relu_open.argtypes = [i, i, sz, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fss_relu_finish.argtypes = [i, i, sz, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        for name in ("fss_sign_mask", "fss_sign_eval", "fss_relu_open", "fss_relu_finish"):
            getattr(L, name).restype = i
        L.fss_eq_mask.argtypes = [i, sz, vp, vp, vp, vp]
        L.fss_eq_masked_eval.argtypes = [i, i, sz, vp, vp, vp, vp, vp]
        L.fss_argmax_diff_mask.argtypes = [i, sz, i, vp, vp, vp, vp]
        L.fss_argmax_count_mask.argtypes = [i, i, sz, i, vp, vp, vp, vp]
        L.fss_maxpool_unroll.argtypes = [sz, i, i, i, i, vp, vp, vp]
        L.fss_mul_open.argtypes = [i, sz, vp, vp, vp, vp, vp, vp, vp]
        L.fss_dot_finish.argtypes = [i, i, sz, i, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        for name in ("fss_eq_mask", "fss_eq_masked_eval", "fss_argmax_diff_mask", "fss_argmax_count_mask", "fss_maxpool_unroll",
                     "fss_mul_open", "fss_dot_finish"):
            getattr(L, name).restype = i
        L.fss_cmp_chunked_key_bytes.argtypes = [i, sz, sz]
        L.fss_cmp_chunked_key_bytes.restype = sz
        L.fss_cmp_eval_streamed.argtypes = [i, i, sz, sz, vp, vp, vp, vp, vp, vp]
        L.fss_cmp_eval_streamed.restype = i
        L.fss_cmp_eval_streamed_static.argtypes = [i, i, sz, sz, vp, vp, vp, vp, vp]
        L.fss_cmp_eval_streamed_static.restype = i
        L.fss_static_staging_bytes.argtypes = []
        L.fss_static_staging_bytes.restype = sz
        L.fss_clock_probe.argtypes = [vp, C.c_uint32, vp]
        L.fss_clock_probe.restype = i
        L.fss_wall_clock_khz.argtypes = []
        L.fss_wall_clock_khz.restype = i
        L.fss_prepare.argtypes = []
        L.fss_prepare.restype = i
        L.fss_quad_layout_below.argtypes = []
        L.fss_quad_layout_below.restype = sz
        L.fss_strerror.argtypes = [i]
        L.fss_strerror.restype = C.c_char_p
        L.fss_last_hip_error.argtypes = []
        L.fss_last_hip_error.restype = i
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        L = lib()
        raise FssError(rc, L.fss_strerror(rc).decode(), L.fss_last_hip_error())


def cmp_key_bytes(n: int, batch: int) -> int:
    return int(lib().fss_cmp_key_bytes(n, batch))


def eq_key_bytes(n: int, batch: int) -> int:
    return int(lib().fss_eq_key_bytes(n, batch))


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _dev(name: str, t, nbytes: int) -> int:
    """Address of a device buffer after checking what a raw pointer cannot say: that it is a
    contiguous GPU tensor of at least `nbytes` bytes.  A kernel launched on a short buffer would
    fault the GPU; here it is a ValueError instead.  None is let through (the C side rejects NULL
    unless the call is empty)."""
    if t is None:
        return 0
    if not getattr(t, "is_cuda", False):
        raise ValueError(f"{name}: expected a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor is not contiguous")
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise ValueError(f"{name}: {have} bytes, the call needs {nbytes}")
    return int(t.data_ptr())


def _host_pinned(name: str, t, nbytes: int) -> int:
    if t is None:
        return 0
    if getattr(t, "is_cuda", True) or not t.is_pinned():
        raise ValueError(f"{name}: expected a pinned host tensor")
    if not t.is_contiguous() or t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{name}: needs {nbytes} contiguous bytes")
    return int(t.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _gen(fn, key_bytes, n, batch, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream):
    kb = key_bytes(n, batch)
    _check(fn(n, batch, _dev("alpha", d_alpha, 4 * batch), _dev("alpha_r", d_alpha_r, 4 * batch), _dev("seed0", d_seed0, 16 * batch),
              _dev("seed1", d_seed1, 16 * batch), _dev("key0", d_key0, kb), _dev("key1", d_key1, kb), _stream(stream)))


def cmp_gen(n: int, batch: int, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream=None) -> None:
    """fss_cmp_gen: device tensors in, both parties' key buffers (uint8 device tensors) out."""
    _gen(lib().fss_cmp_gen, cmp_key_bytes, n, batch, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream)


def eq_gen(n: int, batch: int, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream=None) -> None:
    _gen(lib().fss_eq_gen, eq_key_bytes, n, batch, d_alpha, d_alpha_r, d_seed0, d_seed1, d_key0, d_key1, stream)


def cmp_eval(party: int, n: int, batch: int, d_key, d_x, d_out, stream=None) -> None:
    _check(lib().fss_cmp_eval(party, n, batch, _dev("key", d_key, cmp_key_bytes(n, batch)), _dev("x", d_x, 4 * batch),
                              _dev("out", d_out, 4 * batch), _stream(stream)))


def eq_eval(party: int, n: int, batch: int, d_key, d_x, d_out, stream=None) -> None:
    _check(lib().fss_eq_eval(party, n, batch, _dev("key", d_key, eq_key_bytes(n, batch)), _dev("x", d_x, 4 * batch),
                             _dev("out", d_out, 4 * batch), _stream(stream)))


def sign_mask(n: int, batch: int, d_key, d_y_share, d_masked, stream=None) -> None:
    _check(lib().fss_sign_mask(n, batch, _dev("key", d_key, cmp_key_bytes(n, batch)), _dev("y_share", d_y_share, 4 * batch),
                               _dev("masked", d_masked, 4 * batch), _stream(stream)))


def sign_eval(party: int, n: int, batch: int, d_key, d_masked0, d_masked1, d_out, stream=None) -> None:
    _check(lib().fss_sign_eval(party, n, batch, _dev("key", d_key, cmp_key_bytes(n, batch)), _dev("masked0", d_masked0, 4 * batch),
                               _dev("masked1", d_masked1, 4 * batch), _dev("out", d_out, 4 * batch), _stream(stream)))


def relu_open(party: int, n: int, batch: int, d_key, d_masked0, d_masked1, d_y_share, d_tri_a, d_tri_b, d_delta, d_eps,
              stream=None) -> None:
    w = 4 * batch
    _check(lib().fss_relu_open(party, n, batch, _dev("key", d_key, cmp_key_bytes(n, batch)), _dev("masked0", d_masked0, w),
                               _dev("masked1", d_masked1, w), _dev("y_share", d_y_share, w), _dev("tri_a", d_tri_a, w),
                               _dev("tri_b", d_tri_b, w), _dev("delta", d_delta, w), _dev("eps", d_eps, w), _stream(stream)))


def relu_finish(party: int, n: int, batch: int, d_delta0, d_delta1, d_eps0, d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out,
                stream=None) -> None:
    w = 4 * batch
    _check(lib().fss_relu_finish(party, n, batch, _dev("delta0", d_delta0, w), _dev("delta1", d_delta1, w), _dev("eps0", d_eps0, w),
                                 _dev("eps1", d_eps1, w), _dev("tri_a", d_tri_a, w), _dev("tri_b", d_tri_b, w), _dev("tri_c", d_tri_c, w),
                                 _dev("out", d_out, w), _stream(stream)))


def cmp_chunked_key_bytes(n: int, batch: int, chunk: int) -> int:
    return int(lib().fss_cmp_chunked_key_bytes(n, batch, chunk))


def cmp_eval_streamed(party: int, n: int, batch: int, chunk: int, h_key_chunks, d_x, d_out, d_staging, copy_stream,
                      stream=None) -> None:
    """fss_cmp_eval_streamed: h_key_chunks is a pinned HOST tensor in the chunked layout."""
    _check(lib().fss_cmp_eval_streamed(party, n, batch, chunk, _host_pinned("key_chunks", h_key_chunks, cmp_chunked_key_bytes(n, batch, chunk)),
                                       _dev("x", d_x, 4 * batch), _dev("out", d_out, 4 * batch),
                                       _dev("staging", d_staging, 2 * cmp_key_bytes(n, chunk)), _stream(copy_stream), _stream(stream)))


def static_staging_bytes() -> int:
    return int(lib().fss_static_staging_bytes())


def cmp_eval_streamed_static(party: int, n: int, batch: int, chunk: int, h_key_chunks, d_x, d_out, copy_stream, stream=None) -> None:
    """fss_cmp_eval_streamed_static: as cmp_eval_streamed, staging inside the library (no allocation)."""
    _check(lib().fss_cmp_eval_streamed_static(party, n, batch, chunk, _host_pinned("key_chunks", h_key_chunks, cmp_chunked_key_bytes(n, batch, chunk)),
                                              _dev("x", d_x, 4 * batch), _dev("out", d_out, 4 * batch), _stream(copy_stream), _stream(stream)))


def eq_mask(n: int, batch: int, d_key, d_y_share, d_masked, stream=None) -> None:
    _check(lib().fss_eq_mask(n, batch, _dev("key", d_key, eq_key_bytes(n, batch)), _dev("y_share", d_y_share, 4 * batch),
                             _dev("masked", d_masked, 4 * batch), _stream(stream)))


def eq_masked_eval(party: int, n: int, batch: int, d_key, d_masked0, d_masked1, d_out, stream=None) -> None:
    _check(lib().fss_eq_masked_eval(party, n, batch, _dev("key", d_key, eq_key_bytes(n, batch)), _dev("masked0", d_masked0, 4 * batch),
                                    _dev("masked1", d_masked1, 4 * batch), _dev("out", d_out, 4 * batch), _stream(stream)))


def argmax_diff_mask(n: int, rows: int, m: int, d_cmp_key, d_x_share, d_masked, stream=None) -> None:
    pairs = rows * m * (m - 1)
    _check(lib().fss_argmax_diff_mask(n, rows, m, _dev("cmp_key", d_cmp_key, cmp_key_bytes(n, pairs)), _dev("x_share", d_x_share, 4 * rows * m),
                                      _dev("masked", d_masked, 4 * pairs), _stream(stream)))


def argmax_count_mask(party: int, n: int, rows: int, m: int, d_w_share, d_eq_key, d_masked, stream=None) -> None:
    _check(lib().fss_argmax_count_mask(party, n, rows, m, _dev("w_share", d_w_share, 4 * rows * m * (m - 1)),
                                       _dev("eq_key", d_eq_key, eq_key_bytes(n, rows * m)), _dev("masked", d_masked, 4 * rows * m),
                                       _stream(stream)))


def maxpool_unroll(channels: int, h: int, w: int, k: int, s: int, d_x_share, d_rows, stream=None) -> None:
    windows = ((h - k) // s + 1) * ((w - k) // s + 1) if (s > 0 and h >= k and w >= k) else 0
    _check(lib().fss_maxpool_unroll(channels, h, w, k, s, _dev("x_share", d_x_share, 4 * channels * h * w),
                                    _dev("rows", d_rows, 4 * channels * windows * k * k), _stream(stream)))


def mul_open(n: int, count: int, d_u_share, d_v_share, d_tri_a, d_tri_b, d_delta, d_eps, stream=None) -> None:
    w = 4 * count
    _check(lib().fss_mul_open(n, count, _dev("u_share", d_u_share, w), _dev("v_share", d_v_share, w), _dev("tri_a", d_tri_a, w),
                              _dev("tri_b", d_tri_b, w), _dev("delta", d_delta, w), _dev("eps", d_eps, w), _stream(stream)))


def dot_finish(party: int, n: int, rows: int, m: int, d_delta0, d_delta1, d_eps0, d_eps1, d_tri_a, d_tri_b, d_tri_c, d_out,
               stream=None) -> None:
    w = 4 * rows * m
    _check(lib().fss_dot_finish(party, n, rows, m, _dev("delta0", d_delta0, w), _dev("delta1", d_delta1, w), _dev("eps0", d_eps0, w),
                                _dev("eps1", d_eps1, w), _dev("tri_a", d_tri_a, w), _dev("tri_b", d_tri_b, w), _dev("tri_c", d_tri_c, w),
                                _dev("out", d_out, 4 * rows), _stream(stream)))


def clock_probe(d_ticks, iterations: int, stream=None) -> None:
    """fss_clock_probe: d_ticks is a device tensor of two int64 (shader clocks, wall-clock ticks)."""
    _check(lib().fss_clock_probe(_dev("ticks", d_ticks, 16), iterations, _stream(stream)))


def wall_clock_khz() -> int:
    return int(lib().fss_wall_clock_khz())


def prepare() -> None:
    """fss_prepare: per-device set-up of the current device (kernel attributes), once, ahead of the first call."""
    _check(lib().fss_prepare())


def quad_layout_below() -> int:
    """Batch size below which evaluation on the current device uses the four-lanes-per-element layout."""
    return int(lib().fss_quad_layout_below())
