"""ctypes face of libptchunk.so: the same names as include/ptchunk.h.

Argument marshalling only.  Tensors (torch, device or pinned host) are turned
into raw addresses, Python lists into C arrays, status codes into exceptions.
Every step of the path runs inside the HIP library; if the library is missing
this module raises on first use - there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libptchunk.so")

PT_OK, PT_ERR_INVALID_ARG, PT_ERR_ALIGNMENT, PT_ERR_HIP, PT_ERR_STATE, PT_ERR_UNSUPPORTED, PT_ERR_NOMEM = range(7)
PT_BF16, PT_FP16 = 0, 1
PT_FINALIZE_STRICT, PT_FINALIZE_CARRY = 1, 2

EXPORTS = [
    "pt_version", "pt_status_string", "pt_last_error", "pt_ctx_create", "pt_ctx_destroy", "pt_ctx_set_state",
    "pt_layout_dense", "pt_pack_plan_create", "pt_pack_plan_destroy", "pt_chunk_pack_grads", "pt_chunk_unpack",
    "pt_chunk_grad_sqnorm", "pt_chunk_adamw_step", "pt_stream_reserve", "pt_chunk_stream_step", "pt_step_end",
    "pt_step_report_read", "pt_update_consts_read", "pt_step_override", "pt_calib_copy", "pt_ctx_set_option",
    "pt_layout_grouped", "pt_chunk_size_search", "pt_layout_execution_order", "pt_chunk_host_adamw_step",
    "pt_optim_predict", "pt_optim_choose", "pt_ctx_set_no_decay", "pt_chunk_accum_grads",
    "pt_chunk_grad_sqnorm_noalloc", "pt_calib_adamw_pattern", "pt_stream_status",
]


class pt_segment(C.Structure):
    _fields_ = [("src", C.c_void_p), ("src_off", C.c_uint64), ("len", C.c_uint64),
                ("chunk_off", C.c_uint64), ("chunk", C.c_uint32), ("tensor", C.c_uint32)]


class pt_hparams(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("max_norm", C.c_double)]


class pt_scaler_cfg(C.Structure):
    _fields_ = [("init_scale", C.c_double), ("growth", C.c_double), ("backoff", C.c_double),
                ("growth_interval", C.c_int32), ("reserved", C.c_int32)]


class pt_step_report(C.Structure):
    _fields_ = [("sqnorm", C.c_double), ("norm", C.c_double), ("clip_coef", C.c_double),
                ("loss_scale", C.c_double), ("grad_mult", C.c_float), ("found_inf", C.c_int32),
                ("step", C.c_int32), ("good_steps", C.c_int32)]


class pt_update_consts(C.Structure):
    _fields_ = [("c", C.c_float * 9), ("skip", C.c_int32)]


class pt_optim_rates(C.Structure):
    _fields_ = [("gpu_s_fixed", C.c_double), ("gpu_s_per_elem", C.c_double), ("link_s_fixed", C.c_double),
                ("link_s_per_elem", C.c_double), ("host_s_fixed", C.c_double), ("host_s_per_elem", C.c_double),
                ("stream_contention", C.c_double), ("gpu_serial_share", C.c_double)]


class pt_optim_choice(C.Structure):
    _fields_ = [("n_persist", C.c_uint32), ("n_slots", C.c_uint32), ("mode", C.c_int32), ("reserved", C.c_int32),
                ("t_step", C.c_double), ("t_gpu", C.c_double), ("t_other", C.c_double), ("hbm_bytes", C.c_uint64)]


PT_OPTIM_STREAM, PT_OPTIM_HOST = 0, 1


class PtError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}: {text}")


_lib = None


def lib():
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                               "(python -m paper_2406_08334_amd.build); there is no fallback path")
        # PyTorch ships its own HIP runtime (same SONAME as the system one).  Importing torch
        # first makes this library bind to THAT runtime, so both share one device context and
        # one view of every allocation; loading in the other order would start two runtimes.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int32
        pp = C.POINTER(C.c_void_p)
        L.pt_version.restype = C.c_char_p
        L.pt_version.argtypes = []
        L.pt_status_string.restype = C.c_char_p
        L.pt_status_string.argtypes = [C.c_int]
        L.pt_last_error.restype = C.c_char_p
        L.pt_last_error.argtypes = [vp]
        L.pt_ctx_create.argtypes = [pp, C.c_int, u64, u32, C.POINTER(pt_scaler_cfg)]
        L.pt_ctx_destroy.argtypes = [vp]
        L.pt_ctx_set_state.argtypes = [vp, i32, C.c_double, i32, vp]
        L.pt_layout_dense.argtypes = [C.POINTER(u64), u32, u64, C.POINTER(pt_segment), u32, C.POINTER(u32),
                                      C.POINTER(u32)]
        L.pt_pack_plan_create.argtypes = [vp, C.POINTER(pt_segment), u32, pp]
        L.pt_pack_plan_destroy.argtypes = [vp]
        L.pt_chunk_pack_grads.argtypes = [vp, vp, pp, vp]
        L.pt_chunk_unpack.argtypes = [vp, vp, pp, vp]
        L.pt_chunk_accum_grads.argtypes = [vp, vp, pp, C.c_int, C.c_int, vp]
        L.pt_chunk_grad_sqnorm.argtypes = [vp, pp, u32, u32, C.c_int, vp]
        L.pt_chunk_grad_sqnorm_noalloc.argtypes = [vp, C.c_int, u64, u32, C.c_double, vp, vp, vp]
        L.pt_chunk_adamw_step.argtypes = [vp, C.POINTER(pt_hparams), u32, u32, pp, pp, pp, pp, pp, vp]
        L.pt_stream_reserve.argtypes = [vp, u32]
        L.pt_stream_status.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32)]
        L.pt_chunk_stream_step.argtypes = [vp, C.POINTER(pt_hparams), u32, u32, pp, pp, pp, pp, pp, vp]
        L.pt_step_end.argtypes = [vp, vp]
        L.pt_chunk_host_adamw_step.argtypes = [vp, C.POINTER(pt_hparams), u32, u32, pp, pp, pp, pp, pp, u32, vp]
        L.pt_step_report_read.argtypes = [vp, C.POINTER(pt_step_report), vp]
        L.pt_update_consts_read.argtypes = [vp, C.POINTER(pt_update_consts), vp]
        L.pt_step_override.argtypes = [vp, C.c_float, i32, vp]
        L.pt_calib_copy.argtypes = [vp, vp, u64, vp]
        L.pt_calib_adamw_pattern.argtypes = [vp, u32, u32, vp]
        L.pt_ctx_set_option.argtypes = [vp, C.c_char_p, C.c_int64]
        L.pt_ctx_set_no_decay.argtypes = [vp, C.POINTER(pt_segment), u32]
        dp = C.POINTER(C.c_double)
        L.pt_optim_predict.argtypes = [C.POINTER(pt_optim_rates), u64, u32, u32, C.c_int, dp, dp, dp]
        L.pt_optim_choose.argtypes = [C.POINTER(pt_optim_rates), u64, u32, u64, C.c_int, u32, C.POINTER(pt_optim_choice)]
        L.pt_layout_grouped.argtypes = [C.POINTER(u64), C.POINTER(u32), u32, u64, C.POINTER(pt_segment), u32,
                                        C.POINTER(u32), C.POINTER(u32), C.POINTER(u64)]
        L.pt_layout_execution_order.argtypes = [C.POINTER(u32), u32, u32, C.POINTER(u32)]
        L.pt_chunk_size_search.argtypes = [C.POINTER(u64), C.POINTER(u32), u32, u64, u64, u64, C.POINTER(u64),
                                           C.POINTER(u32), C.POINTER(u64)]
        for name in EXPORTS:
            if name not in ("pt_version", "pt_status_string", "pt_last_error"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


# ---- marshalling helpers ----------------------------------------------------------------

def _addr(x) -> int:
    """Raw address of a torch tensor (device or pinned host), an int, or None."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(items):
    if items is None:
        return None
    arr = (C.c_void_p * max(len(items), 1))()
    for i, t in enumerate(items):
        arr[i] = _addr(t) or None
    return arr


def _stream(stream) -> int:
    """torch.cuda.Stream -> hipStream_t handle; None -> torch's current stream."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def _check(rc: int, where: str, ctx=None):
    if rc != PT_OK:
        text = lib().pt_last_error(ctx).decode()
        raise PtError(rc, where, text)


def hparams(lr, beta1, beta2, eps, weight_decay, max_norm) -> pt_hparams:
    return pt_hparams(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), float(max_norm))


# ---- the calls, same names as the header ------------------------------------------------

def pt_version() -> str:
    return lib().pt_version().decode()


def status_string(status: int) -> str:
    return lib().pt_status_string(int(status)).decode()


def pt_last_error(ctx=None) -> str:
    return lib().pt_last_error(ctx).decode()


def pt_ctx_create(dtype: int, chunk_elems: int, n_chunks: int, scaler: pt_scaler_cfg | None = None):
    out = C.c_void_p()
    rc = lib().pt_ctx_create(C.byref(out), int(dtype), int(chunk_elems), int(n_chunks),
                             C.byref(scaler) if scaler is not None else None)
    _check(rc, "pt_ctx_create")
    return out


def pt_ctx_destroy(ctx):
    _check(lib().pt_ctx_destroy(ctx), "pt_ctx_destroy")


def pt_ctx_set_state(ctx, step: int, loss_scale: float, good_steps: int, stream=None):
    _check(lib().pt_ctx_set_state(ctx, int(step), float(loss_scale), int(good_steps), _stream(stream)),
           "pt_ctx_set_state", ctx)


def pt_layout_dense(tensor_elems, chunk_elems: int):
    """-> (list of pt_segment with src unset, n_chunks).  Host only, no GPU needed."""
    n = len(tensor_elems)
    sizes = (C.c_uint64 * max(n, 1))(*[int(x) for x in tensor_elems])
    nseg, nchunks = C.c_uint32(), C.c_uint32()
    rc = lib().pt_layout_dense(sizes, n, int(chunk_elems), None, 0, C.byref(nseg), C.byref(nchunks))
    _check(rc, "pt_layout_dense")
    segs = (pt_segment * max(nseg.value, 1))()
    rc = lib().pt_layout_dense(sizes, n, int(chunk_elems), segs, nseg.value, C.byref(nseg), C.byref(nchunks))
    _check(rc, "pt_layout_dense")
    return [segs[i] for i in range(nseg.value)], int(nchunks.value)


def pt_pack_plan_create(ctx, segments):
    n = len(segments)
    arr = (pt_segment * max(n, 1))()
    for i, s in enumerate(segments):
        arr[i] = s
    out = C.c_void_p()
    _check(lib().pt_pack_plan_create(ctx, arr, n, C.byref(out)), "pt_pack_plan_create", ctx)
    return out


def pt_pack_plan_destroy(plan):
    _check(lib().pt_pack_plan_destroy(plan), "pt_pack_plan_destroy")


def pt_chunk_pack_grads(ctx, plan, grad_chunks, stream=None):
    _check(lib().pt_chunk_pack_grads(ctx, plan, _ptr_array(grad_chunks), _stream(stream)),
           "pt_chunk_pack_grads", ctx)


def pt_chunk_unpack(ctx, plan, chunks, stream=None):
    _check(lib().pt_chunk_unpack(ctx, plan, _ptr_array(chunks), _stream(stream)), "pt_chunk_unpack", ctx)


def pt_chunk_grad_sqnorm(ctx, grad_chunks, first_chunk: int, n_chunks: int, finalize, stream=None):
    """finalize: False / 0, True / PT_FINALIZE_STRICT, or PT_FINALIZE_CARRY"""
    _check(lib().pt_chunk_grad_sqnorm(ctx, _ptr_array(grad_chunks), int(first_chunk), int(n_chunks),
                                      int(finalize), _stream(stream)), "pt_chunk_grad_sqnorm", ctx)


def pt_chunk_grad_sqnorm_noalloc(grad_arena, dtype: int, chunk_elems: int, n_chunks: int, loss_scale: float,
                                 out_sqnorm_norm, out_found_inf, stream=None):
    """grad_arena: device tensor holding the chunks back to back; out_sqnorm_norm: device float64[2];
    out_found_inf: device int32[1].  Allocates nothing."""
    _check(lib().pt_chunk_grad_sqnorm_noalloc(_addr(grad_arena), int(dtype), int(chunk_elems), int(n_chunks),
                                              float(loss_scale), _addr(out_sqnorm_norm), _addr(out_found_inf),
                                              _stream(stream)), "pt_chunk_grad_sqnorm_noalloc")


def pt_chunk_adamw_step(ctx, hp: pt_hparams, first_chunk: int, n_chunks: int, grad, master, m, v, param16,
                        stream=None):
    _check(lib().pt_chunk_adamw_step(ctx, C.byref(hp), int(first_chunk), int(n_chunks), _ptr_array(grad),
                                     _ptr_array(master), _ptr_array(m), _ptr_array(v), _ptr_array(param16),
                                     _stream(stream)), "pt_chunk_adamw_step", ctx)


def pt_stream_reserve(ctx, n_slots: int):
    _check(lib().pt_stream_reserve(ctx, int(n_slots)), "pt_stream_reserve", ctx)


def pt_stream_status(ctx):
    """-> dict(duplex_tested, duplex_ok, attempts, rebuilds): outcome of pt_stream_reserve's test of its copy
    streams, and how often a serialised step has made pt_chunk_stream_step replace the side streams since."""
    a, b, c, d = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().pt_stream_status(ctx, C.byref(a), C.byref(b), C.byref(c), C.byref(d)), "pt_stream_status", ctx)
    return {"duplex_tested": bool(a.value), "duplex_ok": bool(b.value), "attempts": int(c.value),
            "rebuilds": int(d.value)}


def pt_chunk_stream_step(ctx, hp: pt_hparams, first_chunk: int, n_chunks: int, h_grad, h_master, h_m, h_v,
                         h_param16, stream=None):
    _check(lib().pt_chunk_stream_step(ctx, C.byref(hp), int(first_chunk), int(n_chunks), _ptr_array(h_grad),
                                      _ptr_array(h_master), _ptr_array(h_m), _ptr_array(h_v),
                                      _ptr_array(h_param16), _stream(stream)), "pt_chunk_stream_step", ctx)


def pt_step_end(ctx, stream=None):
    _check(lib().pt_step_end(ctx, _stream(stream)), "pt_step_end", ctx)


def pt_step_report_read(ctx, stream=None) -> pt_step_report:
    out = pt_step_report()
    _check(lib().pt_step_report_read(ctx, C.byref(out), _stream(stream)), "pt_step_report_read", ctx)
    return out


def pt_update_consts_read(ctx, stream=None) -> pt_update_consts:
    out = pt_update_consts()
    _check(lib().pt_update_consts_read(ctx, C.byref(out), _stream(stream)), "pt_update_consts_read", ctx)
    return out


def pt_step_override(ctx, grad_mult: float, found_inf: bool, stream=None):
    _check(lib().pt_step_override(ctx, float(grad_mult), 1 if found_inf else 0, _stream(stream)),
           "pt_step_override", ctx)


def pt_calib_copy(dst, src, nbytes: int, stream=None):
    _check(lib().pt_calib_copy(_addr(dst), _addr(src), int(nbytes), _stream(stream)), "pt_calib_copy")


def pt_calib_adamw_pattern(ctx, first_chunk: int, n_chunks: int, stream=None):
    _check(lib().pt_calib_adamw_pattern(ctx, int(first_chunk), int(n_chunks), _stream(stream)),
           "pt_calib_adamw_pattern", ctx)


def pt_ctx_set_option(ctx, name: str, value: int):
    _check(lib().pt_ctx_set_option(ctx, name.encode(), int(value)), "pt_ctx_set_option", ctx)


PT_NO_GROUP = 0xFFFFFFFF


def _group_array(tensor_group, n):
    if tensor_group is None:
        return None
    return (C.c_uint32 * max(n, 1))(*[PT_NO_GROUP if g is None else int(g) for g in tensor_group])


def pt_layout_execution_order(uses, n_tensors: int):
    """-> tensor indices by first use in the trace `uses`, unused ones behind.  Host only."""
    n = len(uses)
    arr = (C.c_uint32 * max(n, 1))(*[int(u) for u in uses])
    out = (C.c_uint32 * max(int(n_tensors), 1))()
    _check(lib().pt_layout_execution_order(arr, n, int(n_tensors), out), "pt_layout_execution_order")
    return [int(out[i]) for i in range(int(n_tensors))]


def pt_layout_grouped(tensor_elems, tensor_group, chunk_elems: int):
    """-> (list of pt_segment with src unset, n_chunks, waste_elems).  Host only."""
    n = len(tensor_elems)
    sizes = (C.c_uint64 * max(n, 1))(*[int(x) for x in tensor_elems])
    groups = _group_array(tensor_group, n)
    nseg, nchunks, waste = C.c_uint32(), C.c_uint32(), C.c_uint64()
    rc = lib().pt_layout_grouped(sizes, groups, n, int(chunk_elems), None, 0, C.byref(nseg), C.byref(nchunks),
                                 C.byref(waste))
    _check(rc, "pt_layout_grouped")
    segs = (pt_segment * max(nseg.value, 1))()
    rc = lib().pt_layout_grouped(sizes, groups, n, int(chunk_elems), segs, nseg.value, C.byref(nseg),
                                 C.byref(nchunks), C.byref(waste))
    _check(rc, "pt_layout_grouped")
    return [segs[i] for i in range(nseg.value)], int(nchunks.value), int(waste.value)


def pt_chunk_size_search(tensor_elems, tensor_group, min_chunk_elems: int, span_elems: int, step_elems: int):
    """-> (best chunk_elems, n_chunks, waste_elems).  Host only."""
    n = len(tensor_elems)
    sizes = (C.c_uint64 * max(n, 1))(*[int(x) for x in tensor_elems])
    best, nchunks, waste = C.c_uint64(), C.c_uint32(), C.c_uint64()
    rc = lib().pt_chunk_size_search(sizes, _group_array(tensor_group, n), n, int(min_chunk_elems), int(span_elems),
                                    int(step_elems), C.byref(best), C.byref(nchunks), C.byref(waste))
    _check(rc, "pt_chunk_size_search")
    return int(best.value), int(nchunks.value), int(waste.value)


def pt_chunk_host_adamw_step(ctx, hp: pt_hparams, first_chunk: int, n_chunks: int, h_grad, h_master, h_m, h_v,
                             h_param16, n_threads: int, stream=None):
    _check(lib().pt_chunk_host_adamw_step(ctx, C.byref(hp), int(first_chunk), int(n_chunks), _ptr_array(h_grad),
                                          _ptr_array(h_master), _ptr_array(h_m), _ptr_array(h_v),
                                          _ptr_array(h_param16), int(n_threads), _stream(stream)),
           "pt_chunk_host_adamw_step", ctx)


def pt_optim_predict(rates: pt_optim_rates, chunk_elems: int, n_chunks: int, n_persist: int, mode: int):
    """-> (t_gpu, t_other, t_step) in seconds.  Host only."""
    a, b, c = C.c_double(), C.c_double(), C.c_double()
    _check(lib().pt_optim_predict(C.byref(rates), int(chunk_elems), int(n_chunks), int(n_persist), int(mode),
                                  C.byref(a), C.byref(b), C.byref(c)), "pt_optim_predict")
    return a.value, b.value, c.value


def pt_optim_choose(rates: pt_optim_rates, chunk_elems: int, n_chunks: int, hbm_budget_bytes: int, mode: int,
                    n_slots: int = 3) -> pt_optim_choice:
    out = pt_optim_choice()
    _check(lib().pt_optim_choose(C.byref(rates), int(chunk_elems), int(n_chunks), int(hbm_budget_bytes), int(mode),
                                 int(n_slots), C.byref(out)), "pt_optim_choose")
    return out


def pt_ctx_set_no_decay(ctx, segments):
    n = len(segments)
    arr = (pt_segment * max(n, 1))()
    for i, s in enumerate(segments):
        arr[i] = s
    _check(lib().pt_ctx_set_no_decay(ctx, arr, n), "pt_ctx_set_no_decay", ctx)


def pt_chunk_accum_grads(ctx, plan, acc_chunks, overwrite, take_norm, stream=None):
    _check(lib().pt_chunk_accum_grads(ctx, plan, _ptr_array(acc_chunks), int(bool(overwrite)), int(bool(take_norm)),
                                      _stream(stream)), "pt_chunk_accum_grads", ctx)
