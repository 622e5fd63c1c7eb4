"""ctypes/numpy face of the CPU oracle (oracle/oracle.cpp).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the bench's cpu_baseline leg
may import this package; the product package never does, and this package never
imports the product package.  Every function here only marshals numpy arrays into
the C++ routines; all arithmetic lives in oracle.cpp.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ORACLE_SRC_OVERRIDE: build and load another source file instead (tests/oracle_mutation_check.py
# points it at copies of oracle.cpp with one planted mistake each, to see the pins catch it)
_OVERRIDE = os.environ.get("ORACLE_SRC_OVERRIDE")
_SRC = _OVERRIDE or os.path.join(_HERE, "oracle.cpp")
_LIB = (os.path.splitext(_OVERRIDE)[0] + ".so") if _OVERRIDE else os.path.join(_HERE, "liboracle.so")

BF16, FP16 = 0, 1


def build(force: bool = False) -> str:
    """Compile oracle.cpp with g++ (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class Hparams(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("max_norm", C.c_double)]


class ScalerCfg(C.Structure):
    _fields_ = [("init_scale", C.c_double), ("growth", C.c_double), ("backoff", C.c_double),
                ("growth_interval", C.c_int32), ("enabled", C.c_int32)]


class State(C.Structure):
    _fields_ = [("t", C.c_int32), ("good_steps", C.c_int32), ("loss_scale", C.c_double)]


class Report(C.Structure):
    _fields_ = [("sqnorm", C.c_double), ("norm", C.c_double), ("clip_coef", C.c_double),
                ("grad_mult", C.c_double), ("loss_scale_used", C.c_double),
                ("found_inf", C.c_int32), ("t_after", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u16p, f32p, u64p = C.POINTER(C.c_uint16), C.POINTER(C.c_float), C.POINTER(C.c_uint64)
        L.orc_decode16.restype = C.c_float
        L.orc_decode16.argtypes = [C.c_uint16, C.c_int]
        L.orc_encode16_rne.restype = C.c_uint16
        L.orc_encode16_rne.argtypes = [C.c_float, C.c_int]
        L.orc_decode16_array.restype = None
        L.orc_decode16_array.argtypes = [u16p, f32p, C.c_uint64, C.c_int]
        L.orc_encode16_array.restype = None
        L.orc_encode16_array.argtypes = [f32p, u16p, C.c_uint64, C.c_int]
        L.orc_pack_dense.restype = C.c_int64
        L.orc_pack_dense.argtypes = [C.POINTER(u16p), u64p, C.c_uint32, C.c_uint64, u16p, C.c_uint64]
        L.orc_unpack_dense.restype = C.c_int64
        L.orc_unpack_dense.argtypes = [u16p, C.c_uint64, C.c_uint64, C.POINTER(u16p), u64p, C.c_uint32]
        L.orc_pack_segments.restype = None
        L.orc_pack_segments.argtypes = [C.POINTER(u16p), u64p, u64p, C.POINTER(C.c_uint32), u64p, C.c_uint32,
                                        C.c_uint64, u16p]
        L.orc_found_nonfinite.restype = C.c_int32
        L.orc_found_nonfinite.argtypes = [u16p, C.c_uint64, C.c_int]
        L.orc_sqnorm.restype = C.c_double
        L.orc_sqnorm.argtypes = [u16p, C.c_uint64, C.c_int, C.c_double, C.c_uint64, C.c_int]
        L.orc_clip_coef.restype = C.c_double
        L.orc_clip_coef.argtypes = [C.c_double, C.c_double]
        L.orc_adamw_f64.restype = None
        u8p = C.POINTER(C.c_uint8)
        L.orc_adamw_f64.argtypes = [C.POINTER(Hparams), C.c_int32, C.c_double, u16p, f32p, f32p, f32p,
                                    u16p, C.c_uint64, C.c_int, C.c_int, u8p]
        L.orc_consts_f32.restype = None
        L.orc_consts_f32.argtypes = [C.POINTER(Hparams), C.c_int32, C.c_double, f32p]
        L.orc_adamw_f32seq.restype = None
        L.orc_adamw_f32seq.argtypes = [f32p, u16p, f32p, f32p, f32p, u16p, C.c_uint64, C.c_int, C.c_int, u8p]
        L.orc_step.restype = None
        L.orc_step.argtypes = [C.POINTER(Hparams), C.POINTER(ScalerCfg), C.POINTER(State), u16p, f32p,
                               f32p, f32p, u16p, C.c_uint64, C.c_uint64, C.c_int, C.c_int, C.c_int,
                               C.POINTER(Report), u8p]
        L.orc_accum_f32.restype = None
        L.orc_accum_f32.argtypes = [u16p, C.c_uint64, C.c_int, C.c_int, f32p]
        L.orc_found_nonfinite_f32.restype = C.c_int32
        L.orc_found_nonfinite_f32.argtypes = [f32p, C.c_uint64]
        L.orc_sqnorm_f32.restype = C.c_double
        L.orc_sqnorm_f32.argtypes = [f32p, C.c_uint64, C.c_double, C.c_uint64, C.c_int]
        L.orc_adamw_f64_g32.restype = None
        L.orc_adamw_f64_g32.argtypes = [C.POINTER(Hparams), C.c_int32, C.c_double, f32p, f32p, f32p, f32p,
                                        u16p, C.c_uint64, C.c_int, C.c_int, u8p]
        L.orc_adamw_f32seq_g32.restype = None
        L.orc_adamw_f32seq_g32.argtypes = [f32p, f32p, f32p, f32p, f32p, u16p, C.c_uint64, C.c_int, C.c_int, u8p]
        L.orc_step_g32.restype = None
        L.orc_step_g32.argtypes = [C.POINTER(Hparams), C.POINTER(ScalerCfg), C.POINTER(State), f32p, f32p,
                                   f32p, f32p, u16p, C.c_uint64, C.c_uint64, C.c_int, C.c_int, C.c_int,
                                   C.POINTER(Report), u8p]
        L.orc_hardware_threads.restype = C.c_int
        L.orc_hardware_threads.argtypes = []
        _lib = L
    return _lib


def _u16(a):
    assert isinstance(a, np.ndarray) and a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint16))


def _f32(a):
    assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


def hardware_threads() -> int:
    return int(lib().orc_hardware_threads())


def decode16(words: np.ndarray, dtype: int) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint16)
    out = np.empty(words.shape, dtype=np.float32)
    lib().orc_decode16_array(_u16(words), _f32(out), words.size, dtype)
    return out


def encode16_rne(x: np.ndarray, dtype: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_encode16_array(_f32(x), _u16(out), x.size, dtype)
    return out


def pack_dense(tensors, S: int, n_chunks: int | None = None) -> np.ndarray:
    """Concatenate 16-bit tensors into ceil(N/S) chunks of S words -> array [C, S]."""
    tensors = [np.ascontiguousarray(t, dtype=np.uint16).reshape(-1) for t in tensors]
    total = sum(t.size for t in tensors)
    need = max(1, -(-total // S)) if total else 0
    n_chunks = need if n_chunks is None else n_chunks
    chunks = np.full((n_chunks, S), 0xDEAD, dtype=np.uint16)  # the oracle must overwrite all of it
    ptrs = (C.POINTER(C.c_uint16) * len(tensors))(*[_u16(t) for t in tensors])
    elems = (C.c_uint64 * len(tensors))(*[t.size for t in tensors])
    got = lib().orc_pack_dense(ptrs, elems, len(tensors), S, _u16(chunks), n_chunks)
    if got < 0:
        raise ValueError("n_chunks too small")
    if total == 0:
        chunks[...] = 0
    return chunks


def pack_segments(segments, chunks: np.ndarray):
    """segments: iterable of (tensor words, src_off, len, chunk, chunk_off); chunks: uint16 [C, S], changed in place."""
    segs = [(np.ascontiguousarray(t, dtype=np.uint16).reshape(-1), int(so), int(n), int(c), int(co))
            for t, so, n, c, co in segments]
    assert chunks.dtype == np.uint16 and chunks.flags.c_contiguous and chunks.ndim == 2
    C_, S = chunks.shape
    for t, so, n, c, co in segs:
        assert so + n <= t.size and c < C_ and co + n <= S
    k = len(segs)
    ptrs = (C.POINTER(C.c_uint16) * max(k, 1))(*[_u16(t) for t, *_ in segs])
    arr = lambda vals, ct: (ct * max(k, 1))(*vals)
    lib().orc_pack_segments(ptrs, arr([s[1] for s in segs], C.c_uint64), arr([s[2] for s in segs], C.c_uint64),
                            arr([s[3] for s in segs], C.c_uint32), arr([s[4] for s in segs], C.c_uint64), k, S,
                            _u16(chunks))


def unpack_dense(chunks: np.ndarray, sizes) -> list:
    chunks = np.ascontiguousarray(chunks, dtype=np.uint16)
    n_chunks, S = chunks.shape
    outs = [np.empty(int(s), dtype=np.uint16) for s in sizes]
    ptrs = (C.POINTER(C.c_uint16) * len(outs))(*[_u16(t) for t in outs])
    elems = (C.c_uint64 * len(outs))(*[t.size for t in outs])
    got = lib().orc_unpack_dense(_u16(chunks), S, n_chunks, ptrs, elems, len(outs))
    if got < 0:
        raise ValueError("chunks too small for the tensor list")
    return outs


def found_nonfinite(g16: np.ndarray, dtype: int) -> bool:
    g16 = np.ascontiguousarray(g16, dtype=np.uint16).reshape(-1)
    return bool(lib().orc_found_nonfinite(_u16(g16), g16.size, dtype))


def sqnorm(g16: np.ndarray, dtype: int, loss_scale: float = 1.0, block: int = 0, threads: int = 1) -> float:
    g16 = np.ascontiguousarray(g16, dtype=np.uint16).reshape(-1)
    return float(lib().orc_sqnorm(_u16(g16), g16.size, dtype, float(loss_scale), int(block), int(threads)))


def clip_coef(norm: float, max_norm: float) -> float:
    return float(lib().orc_clip_coef(float(norm), float(max_norm)))


def consts_f32(hp: Hparams, t: int, grad_mult: float) -> np.ndarray:
    c = np.empty(9, dtype=np.float32)
    lib().orc_consts_f32(C.byref(hp), int(t), float(grad_mult), _f32(c))
    return c


def _u8_or_null(a, n):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == np.uint8 and a.flags.c_contiguous and a.size == n
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def adamw_f64(hp: Hparams, t: int, grad_mult: float, g16, w, m, v, p16, dtype: int, threads: int = 1,
              no_decay=None):
    """In-place fp64-evaluated AdamW on flat arrays (w, m, v float32; g16, p16 uint16).
    no_decay: optional uint8 array, non-zero = that element is not decayed."""
    n = w.size
    assert g16.size == n and m.size == n and v.size == n and p16.size == n
    lib().orc_adamw_f64(C.byref(hp), int(t), float(grad_mult), _u16(g16), _f32(w), _f32(m), _f32(v),
                        _u16(p16), n, dtype, int(threads), _u8_or_null(no_decay, n))


def adamw_f32seq(consts: np.ndarray, g16, w, m, v, p16, dtype: int, threads: int = 1, no_decay=None):
    """In-place AdamW in the fp32 operation sequence, driven by the nine fp32 constants."""
    n = w.size
    assert g16.size == n and m.size == n and v.size == n and p16.size == n
    consts = np.ascontiguousarray(consts, dtype=np.float32)
    assert consts.size == 9
    lib().orc_adamw_f32seq(_f32(consts), _u16(g16), _f32(w), _f32(m), _f32(v), _u16(p16), n, dtype,
                           int(threads), _u8_or_null(no_decay, n))


def step(hp: Hparams, sc: ScalerCfg | None, st: State, g16, w, m, v, p16, S: int, dtype: int,
         use_f32seq: bool = False, threads: int = 1, no_decay=None) -> Report:
    """One whole optimizer step (scan, norm, clip, update or skip, loss-scale machine)."""
    n = w.size
    assert g16.size == n and m.size == n and v.size == n and p16.size == n
    rep = Report()
    lib().orc_step(C.byref(hp), C.byref(sc) if sc is not None else None, C.byref(st), _u16(g16),
                   _f32(w), _f32(m), _f32(v), _u16(p16), n, int(S), dtype, int(bool(use_f32seq)),
                   int(threads), C.byref(rep), _u8_or_null(no_decay, n))
    return rep


def new_state(sc: ScalerCfg | None) -> State:
    return State(0, 0, float(sc.init_scale) if (sc is not None and sc.enabled) else 1.0)


# ---- gradient accumulation in fp32 (micro-batches) ----------------------------------------

def accum_f32(src16: np.ndarray, acc: np.ndarray, dtype: int, overwrite: bool = False):
    """acc (float32, in place) = [acc +] decode(src16), element by element."""
    src16 = np.ascontiguousarray(src16, dtype=np.uint16).reshape(-1)
    assert acc.size == src16.size
    lib().orc_accum_f32(_u16(src16), src16.size, dtype, int(bool(overwrite)), _f32(acc))


def found_nonfinite_f32(g32: np.ndarray) -> bool:
    return bool(lib().orc_found_nonfinite_f32(_f32(g32), g32.size))


def sqnorm_f32(g32: np.ndarray, loss_scale: float = 1.0, block: int = 0, threads: int = 1) -> float:
    return float(lib().orc_sqnorm_f32(_f32(g32), g32.size, float(loss_scale), int(block), int(threads)))


def adamw_f64_g32(hp: Hparams, t: int, grad_mult: float, g32, w, m, v, p16, dtype: int, threads: int = 1,
                  no_decay=None):
    n = w.size
    assert g32.size == n and m.size == n and v.size == n and p16.size == n
    lib().orc_adamw_f64_g32(C.byref(hp), int(t), float(grad_mult), _f32(g32), _f32(w), _f32(m), _f32(v),
                            _u16(p16), n, dtype, int(threads), _u8_or_null(no_decay, n))


def adamw_f32seq_g32(consts: np.ndarray, g32, w, m, v, p16, dtype: int, threads: int = 1, no_decay=None):
    n = w.size
    assert g32.size == n and m.size == n and v.size == n and p16.size == n
    consts = np.ascontiguousarray(consts, dtype=np.float32)
    assert consts.size == 9
    lib().orc_adamw_f32seq_g32(_f32(consts), _f32(g32), _f32(w), _f32(m), _f32(v), _u16(p16), n, dtype,
                               int(threads), _u8_or_null(no_decay, n))


def step_g32(hp: Hparams, sc: ScalerCfg | None, st: State, g32, w, m, v, p16, S: int, dtype: int,
             use_f32seq: bool = False, threads: int = 1, no_decay=None) -> Report:
    n = w.size
    assert g32.size == n and m.size == n and v.size == n and p16.size == n
    rep = Report()
    lib().orc_step_g32(C.byref(hp), C.byref(sc) if sc is not None else None, C.byref(st), _f32(g32),
                       _f32(w), _f32(m), _f32(v), _u16(p16), n, int(S), dtype, int(bool(use_f32seq)),
                       int(threads), C.byref(rep), _u8_or_null(no_decay, n))
    return rep
