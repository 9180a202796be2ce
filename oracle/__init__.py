"""CPU oracle for the SSM-layer prefill (token-by-token recurrence in fp64) and
for the causal convolution in front of it.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this package;
tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no
code with the GPU library.  The arithmetic lives in `ssm_oracle.c` and
`conv_oracle.c`; this file only builds them with gcc, loads them with ctypes
and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssm_oracle.c")
_LIB = os.path.join(_HERE, "libssm_oracle.so")
_CONV_SRC = os.path.join(_HERE, "conv_oracle.c")
_CONV_LIB = os.path.join(_HERE, "libconv_oracle.so")
_lib = None
_conv_lib = None


def _compile(src: str, lib: str, force: bool) -> None:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", lib, src, "-lm"]
        subprocess.run(cmd, check=True)


def build(force: bool = False) -> str:
    """Compile the oracles with gcc (no fast-math, no contraction)."""
    _compile(_SRC, _LIB, force)
    _compile(_CONV_SRC, _CONV_LIB, force)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_ssm_prefill.restype = ctypes.c_int
        lib.oracle_ssm_prefill.argtypes = [
            ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            f32p, f32p, f32p, f32p, f32p, f32p,
            ctypes.c_int, i32p, ctypes.POINTER(f64p), i32p, i32p,
            f64p, f64p, ctypes.c_int]
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _f32(a) -> np.ndarray:
    """Exact upcast to contiguous float32 (bf16 and fp32 inputs are both
    representable); accepts numpy arrays and CPU torch tensors."""
    if hasattr(a, "detach"):
        a = a.detach().to("cpu").float().numpy()
    return np.ascontiguousarray(a, dtype=np.float32)


def ssm_prefill_oracle(x, dt, A, B, C, D, cu_seqlens, init_states: Optional[Sequence] = None,
                       ckpt_pos: Optional[List[List[int]]] = None, *, want_y: bool = True,
                       nthreads: Optional[int] = None):
    """Run the recurrence.

    x [T,H,P], dt [T,H], A [H], B/C [T,G,N], D [H]; `init_states` is None or a
    list with one entry per sequence (None = zeros, else [H,P,N], converted
    exactly to double); `ckpt_pos` lists, per sequence, ascending token counts.

    Returns (y, states): y is float64 [T,H,P] (None if want_y is False) and
    states is float64 [n_ckpt,H,P,N] in sequence-major checkpoint order.
    """
    lib = _load()
    x, dt, A, B, C, D = (_f32(v) for v in (x, dt, A, B, C, D))
    T, H, P = x.shape
    G, N = B.shape[1], B.shape[2]
    assert dt.shape == (T, H) and A.shape == (H,) and D.shape == (H,)
    assert B.shape == (T, G, N) and C.shape == (T, G, N)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    batch = cu.shape[0] - 1
    ckpt_pos = ckpt_pos if ckpt_pos is not None else [[] for _ in range(batch)]
    assert len(ckpt_pos) == batch
    cu_ck = np.zeros(batch + 1, dtype=np.int32)
    for i, c in enumerate(ckpt_pos):
        cu_ck[i + 1] = cu_ck[i] + len(c)
    flat = np.asarray([p for c in ckpt_pos for p in c] or [0], dtype=np.int32)
    n_ckpt = int(cu_ck[-1])

    f64p = ctypes.POINTER(ctypes.c_double)
    keep = []
    init_arr = None
    if init_states is not None:
        assert len(init_states) == batch
        init_arr = (f64p * max(batch, 1))()
        for i, s in enumerate(init_states):
            if s is None:
                init_arr[i] = None
            else:
                if hasattr(s, "detach"):
                    s = s.detach().to("cpu").double().numpy()
                s64 = np.ascontiguousarray(s, dtype=np.float64)
                assert s64.shape == (H, P, N)
                keep.append(s64)
                init_arr[i] = s64.ctypes.data_as(f64p)

    y = np.empty((T, H, P), dtype=np.float64) if want_y else None
    states = np.zeros((max(n_ckpt, 1), H, P, N), dtype=np.float64)
    nthreads = nthreads or max_threads()

    def p32(a):
        return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))

    def pi(a):
        return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))

    rc = lib.oracle_ssm_prefill(
        T, H, P, N, G, p32(x), p32(dt), p32(A), p32(B), p32(C), p32(D),
        batch, pi(cu), init_arr, pi(cu_ck), pi(flat),
        y.ctypes.data_as(f64p) if want_y else None,
        states.ctypes.data_as(f64p), int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_ssm_prefill rejected its arguments (code {rc})")
    return y, states[:n_ckpt]


def _load_conv():
    global _conv_lib
    if _conv_lib is None:
        build()
        lib = ctypes.CDLL(_CONV_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_conv1d_prefill.restype = ctypes.c_int
        lib.oracle_conv1d_prefill.argtypes = [
            ctypes.c_int64, ctypes.c_int, ctypes.c_int, f32p, f32p, f32p,
            ctypes.c_int, i32p, ctypes.POINTER(f64p), i32p, i32p, ctypes.c_int, f64p, f64p]
        _conv_lib = lib
    return _conv_lib


def conv1d_prefill_oracle(xin, weight, bias, cu_seqlens, init_states: Optional[Sequence] = None,
                          ckpt_pos: Optional[List[List[int]]] = None, *, silu: bool = True):
    """Causal depthwise convolution with cached-state resume.

    xin [T,C], weight [C,K] (weight[:, K-1] multiplies the current token), bias
    [C] or None; `init_states` is None or one entry per sequence (None = zeros,
    else [C,K]: the last K inputs of the cached prefix, oldest first);
    `ckpt_pos` lists, per sequence, ascending token counts.

    Returns (out, states): float64 [T,C] and float64 [n_ckpt,C,K].
    """
    lib = _load_conv()
    xin, weight = _f32(xin), _f32(weight)
    T, C = xin.shape
    K = weight.shape[1]
    assert weight.shape == (C, K)
    b = _f32(bias) if bias is not None else None
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    batch = cu.shape[0] - 1
    ckpt_pos = ckpt_pos if ckpt_pos is not None else [[] for _ in range(batch)]
    assert len(ckpt_pos) == batch
    cu_ck = np.zeros(batch + 1, dtype=np.int32)
    for i, c in enumerate(ckpt_pos):
        cu_ck[i + 1] = cu_ck[i] + len(c)
    flat = np.asarray([p for c in ckpt_pos for p in c] or [0], dtype=np.int32)
    n_ckpt = int(cu_ck[-1])
    f64p = ctypes.POINTER(ctypes.c_double)
    f32p = ctypes.POINTER(ctypes.c_float)
    i32p = ctypes.POINTER(ctypes.c_int32)
    keep = []
    init_arr = None
    if init_states is not None:
        assert len(init_states) == batch
        init_arr = (f64p * max(batch, 1))()
        for i, s in enumerate(init_states):
            if s is None:
                init_arr[i] = None
            else:
                if hasattr(s, "detach"):
                    s = s.detach().to("cpu").double().numpy()
                s64 = np.ascontiguousarray(s, dtype=np.float64)
                assert s64.shape == (C, K)
                keep.append(s64)
                init_arr[i] = s64.ctypes.data_as(f64p)
    out = np.empty((T, C), dtype=np.float64)
    states = np.zeros((max(n_ckpt, 1), C, K), dtype=np.float64)
    rc = lib.oracle_conv1d_prefill(
        T, C, K, xin.ctypes.data_as(f32p), weight.ctypes.data_as(f32p),
        b.ctypes.data_as(f32p) if b is not None else None, batch, cu.ctypes.data_as(i32p), init_arr,
        cu_ck.ctypes.data_as(i32p), flat.ctypes.data_as(i32p), 1 if silu else 0,
        out.ctypes.data_as(f64p), states.ctypes.data_as(f64p))
    if rc != 0:
        raise ValueError(f"oracle_conv1d_prefill rejected its arguments (code {rc})")
    return out, states[:n_ckpt]
