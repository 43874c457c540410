"""Thin ctypes binding of include/psx.h: argument marshalling only.

Every function has the name of the C entry point it calls.  Device and pinned
buffers may be given as torch tensors (their data_ptr() is taken) or as plain
integer addresses.  A negative status raises PsxError with the library's
message.  The native library is required: if libpsx.so is missing or does not
load, the first call raises; nothing here computes anything on its own.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpsx.so")

PSX_OK, PSX_EINVAL, PSX_ETOOLARGE, PSX_ECAP, PSX_EALIGN, PSX_EHIP, PSX_ENOSTAGING, PSX_ECAPTURE = 0, -1, -2, -3, -4, -5, -6, -7
PSX_LAYOUT_STRICT = 1
PSX_F16, PSX_F32 = 1, 2
PSX_PACK_CHECK_OVERFLOW = 1
PSX_LOC_HBM, PSX_LOC_HOST = 0, 1
PSX_EXEC_GPU, PSX_EXEC_CPU = 0, 1
PSX_STEP_USE_FLAG, PSX_STEP_CHECK_FIRST, PSX_STEP_DEVICE_STATE = 1, 2, 4
PSX_TUNE_ADAM_BLOCKS_PER_CU, PSX_TUNE_ADAM_UNROLL, PSX_TUNE_NONTEMPORAL, PSX_TUNE_COPY_BLOCKS_PER_CU = 1, 2, 3, 4
PSX_TUNE_ADAM_THREADS, PSX_TUNE_ADAM_WG_PER_CU, PSX_TUNE_COPY_UNROLL = 5, 6, 7
PSX_TUNE_HOST_MODE, PSX_TUNE_HOST_GRID, PSX_TUNE_HOST_UNROLL = 8, 9, 10
PSX_TUNE_CPU_THREADS, PSX_TUNE_CPU_TILE_ELEMS, PSX_TUNE_CPU_ISA = 11, 12, 13
PSX_TUNE_COPY_THREADS = 14
PSX_TUNE_FUSED_UNPACK = 15
PSX_ADVANCE_CLEAR_FLAGS = 1
PSX_NOALLOC_MAX_CHUNKS, PSX_NOALLOC_SCRATCH_BYTES = 1024, 262144

EXPORTS = [
    "psx_last_error", "psx_chunk_layout", "psx_ctx_create", "psx_ctx_destroy", "psx_pack", "psx_unpack",
    "psx_overflow_check", "psx_overflow_reset", "psx_overflow_read", "psx_chunk_adam_step",
    "psx_loss_scale_update", "psx_ctx_set_tuning", "psx_ctx_set_profiling", "psx_ctx_get_timing",
    "psx_copy_bytes", "psx_measure_link", "psx_pinned_alloc", "psx_pinned_free", "psx_plan_residency",
    "psx_chunk_size_search", "psx_chunk_adam_step_noalloc", "psx_adam_step_scalars",
    "psx_step_state_init", "psx_step_state_advance", "psx_step_state_read", "psx_chunk_adam_step_unpack",
]


class PsxError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"psx status {code}: {msg}")
        self.code = code


class psx_slot(C.Structure):
    _fields_ = [("chunk", C.c_uint32), ("reserved", C.c_uint32), ("offset", C.c_uint64), ("numel", C.c_uint64)]


class psx_ctx_config(C.Structure):
    _fields_ = [("max_chunks", C.c_uint64), ("max_tensors", C.c_uint64), ("staging_tile_elems", C.c_uint64),
                ("staging_slots", C.c_uint32), ("reserved", C.c_uint32)]


class psx_adam_hyper(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("loss_scale", C.c_double), ("step", C.c_uint64),
                ("adamw_mode", C.c_uint32), ("reserved", C.c_uint32)]


class psx_chunk(C.Structure):
    _fields_ = [("g16", C.c_void_p), ("p16", C.c_void_p), ("p32", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("p32_host", C.c_void_p), ("m_host", C.c_void_p), ("v_host", C.c_void_p), ("used", C.c_uint64),
                ("loc_in", C.c_uint8), ("loc_out", C.c_uint8), ("exec", C.c_uint8), ("reserved", C.c_uint8 * 5)]


class psx_scaler(C.Structure):
    _fields_ = [("scale", C.c_float), ("growth_interval", C.c_uint32), ("good_steps", C.c_uint32),
                ("reserved", C.c_uint32), ("step", C.c_uint64)]


class psx_timing(C.Structure):
    _fields_ = [("pack_ms", C.c_float), ("check_ms", C.c_float), ("adam_ms", C.c_float), ("spill_ms", C.c_float),
                ("adam_elems", C.c_uint64), ("spill_elems", C.c_uint64), ("h2d_bytes", C.c_uint64),
                ("d2h_bytes", C.c_uint64), ("cpu_ms", C.c_float), ("cpu_threads", C.c_uint32),
                ("cpu_elems", C.c_uint64), ("unpack_ms", C.c_float), ("reserved", C.c_uint32)]


class psx_link_rates(C.Structure):
    _fields_ = [("h2d_alone", C.c_double), ("d2h_alone", C.c_double), ("each_way_both", C.c_double)]


_lib = None


def lib():
    """Load libpsx.so (after torch, so that both use the one HIP runtime torch ships)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2108_05818_amd.build` "
                          "(there is no CPU fallback)")
    import torch  # noqa: F401  (loads libamdhip64 first)
    L = C.CDLL(LIB_PATH)
    vp, u32, u64, sz = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t
    L.psx_last_error.restype = C.c_char_p
    L.psx_last_error.argtypes = []
    sigs = {
        "psx_chunk_layout": [vp, sz, u64, u32, vp, vp, sz, C.POINTER(sz)],
        "psx_ctx_create": [C.POINTER(psx_ctx_config), C.POINTER(vp)],
        "psx_ctx_destroy": [vp],
        "psx_pack": [vp, u32, vp, vp, sz, vp, sz, u64, u32, vp],
        "psx_unpack": [vp, u32, vp, vp, sz, vp, sz, u64, u32, vp],
        "psx_overflow_check": [vp, vp, vp, sz, vp, vp, vp],
        "psx_overflow_reset": [vp, vp],
        "psx_overflow_read": [vp, vp, sz, vp, vp],
        "psx_chunk_adam_step": [vp, vp, sz, C.POINTER(psx_adam_hyper), u32, vp],
        "psx_chunk_adam_step_noalloc": [vp, sz, C.POINTER(psx_adam_hyper), u32, vp, vp],
        "psx_chunk_adam_step_unpack": [vp, vp, sz, C.POINTER(psx_adam_hyper), u32, vp, vp, sz, u64, vp],
        "psx_adam_step_scalars": [C.POINTER(psx_adam_hyper), vp],
        "psx_step_state_init": [vp, C.POINTER(psx_adam_hyper), C.POINTER(psx_scaler), vp],
        "psx_step_state_advance": [vp, u32, vp],
        "psx_step_state_read": [vp, C.POINTER(psx_scaler), C.POINTER(u32), C.POINTER(u64), vp],
        "psx_loss_scale_update": [C.POINTER(psx_scaler), u32],
        "psx_ctx_set_tuning": [vp, u32, C.c_int64],
        "psx_ctx_set_profiling": [vp, C.c_int32],
        "psx_ctx_get_timing": [vp, C.POINTER(psx_timing)],
        "psx_copy_bytes": [vp, vp, vp, u64, vp],
        "psx_measure_link": [vp, u64, u32, C.POINTER(psx_link_rates)],
        "psx_pinned_alloc": [u64, C.POINTER(vp)],
        "psx_pinned_free": [vp],
        "psx_plan_residency": [vp, sz, u64, u64, vp, C.POINTER(u64)],
        "psx_chunk_size_search": [vp, sz, u64, u64, u64, u32, u64, C.POINTER(u64), C.POINTER(C.c_double),
                                  C.POINTER(sz)],
    }
    for name, args in sigs.items():
        f = getattr(L, name)
        f.restype = C.c_int32
        f.argtypes = args
    _lib = L
    return L


def _ok(rc):
    if rc != 0:
        raise PsxError(rc, lib().psx_last_error().decode())


def _addr(x):
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return x.data_ptr()


def ptr_array(items):
    """Host array of addresses from tensors / ints / None."""
    return (C.c_void_p * max(len(items), 1))(*[_addr(x) for x in items])


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return _addr(stream) if not hasattr(stream, "cuda_stream") else stream.cuda_stream


def psx_last_error():
    return lib().psx_last_error().decode()


def psx_chunk_layout(numel, chunk_elems, flags=0):
    """-> (slots: ctypes array of psx_slot, used: list[int])."""
    n = len(numel)
    arr = (C.c_uint64 * max(n, 1))(*numel)
    nch = C.c_size_t(0)
    _ok(lib().psx_chunk_layout(arr, n, chunk_elems, flags, None, None, 0, C.byref(nch)))
    slots = (psx_slot * max(n, 1))()
    used = (C.c_uint64 * nch.value)()
    _ok(lib().psx_chunk_layout(arr, n, chunk_elems, flags, slots, used, nch.value, C.byref(nch)))
    return slots, list(used)


def psx_ctx_create(max_chunks, max_tensors, staging_tile_elems=0, staging_slots=3):
    cfg = psx_ctx_config(max_chunks, max_tensors, staging_tile_elems, staging_slots, 0)
    out = C.c_void_p(0)
    _ok(lib().psx_ctx_create(C.byref(cfg), C.byref(out)))
    return out


def psx_ctx_destroy(ctx):
    _ok(lib().psx_ctx_destroy(ctx))


def psx_pack(ctx, dtype, tensors, slots, chunks, chunk_elems, flags=0, stream=None, n=None):
    n = len(tensors) if n is None else n
    t = tensors if isinstance(tensors, C.Array) else ptr_array(tensors)
    c = chunks if isinstance(chunks, C.Array) else ptr_array(chunks)
    _ok(lib().psx_pack(ctx, dtype, t, slots, n, c, len(chunks), chunk_elems, flags, _stream(stream)))


def psx_unpack(ctx, dtype, tensors, slots, chunks, chunk_elems, flags=0, stream=None, n=None):
    n = len(tensors) if n is None else n
    t = tensors if isinstance(tensors, C.Array) else ptr_array(tensors)
    c = chunks if isinstance(chunks, C.Array) else ptr_array(chunks)
    _ok(lib().psx_unpack(ctx, dtype, t, slots, n, c, len(chunks), chunk_elems, flags, _stream(stream)))


def psx_overflow_check(ctx, g16_chunks, used, stream=None, read=True):
    """-> (flag, per_chunk list) when read, else None (asynchronous)."""
    n = len(g16_chunks)
    c = g16_chunks if isinstance(g16_chunks, C.Array) else ptr_array(g16_chunks)
    u = (C.c_uint64 * max(n, 1))(*used)
    if not read:
        _ok(lib().psx_overflow_check(ctx, c, u, n, None, None, _stream(stream)))
        return None
    per = (C.c_uint32 * max(n, 1))()
    flag = C.c_uint32(0)
    _ok(lib().psx_overflow_check(ctx, c, u, n, per, C.byref(flag), _stream(stream)))
    return flag.value, list(per)[:n]


def psx_overflow_reset(ctx, stream=None):
    _ok(lib().psx_overflow_reset(ctx, _stream(stream)))


def psx_overflow_read(ctx, n_chunks=0, stream=None):
    per = (C.c_uint32 * max(n_chunks, 1))()
    flag = C.c_uint32(0)
    _ok(lib().psx_overflow_read(ctx, per if n_chunks else None, n_chunks, C.byref(flag), _stream(stream)))
    return flag.value, list(per)[:n_chunks]


def make_hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, adamw_mode=0, step=1, loss_scale=1.0):
    return psx_adam_hyper(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
                          float(loss_scale), int(step), int(adamw_mode), 0)


def make_chunks(specs):
    """specs: list of dicts with keys g16, p16, used and (p32, m, v) and/or (p32_host, m_host, v_host),
    loc_in, loc_out.  Returns a ctypes array of psx_chunk."""
    arr = (psx_chunk * max(len(specs), 1))()
    for i, s in enumerate(specs):
        a = arr[i]
        for k in ("g16", "p16", "p32", "m", "v", "p32_host", "m_host", "v_host"):
            setattr(a, k, _addr(s.get(k)) or None)
        a.used = int(s["used"])
        a.loc_in = int(s.get("loc_in", PSX_LOC_HBM))
        a.loc_out = int(s.get("loc_out", a.loc_in))
        a.exec = int(s.get("exec", PSX_EXEC_GPU))
    return arr


def psx_chunk_adam_step(ctx, chunks, hyper, flags=0, stream=None, n_chunks=None):
    n = len(chunks) if n_chunks is None else n_chunks
    _ok(lib().psx_chunk_adam_step(ctx, chunks, n, C.byref(hyper), flags, _stream(stream)))


def psx_chunk_adam_step_unpack(ctx, chunks, hyper, flags, p16_tensors, slots, chunk_elems, stream=None, n_chunks=None, n=None):
    nc = len(chunks) if n_chunks is None else n_chunks
    n = len(p16_tensors) if n is None else n
    t = p16_tensors if isinstance(p16_tensors, C.Array) else ptr_array(p16_tensors)
    _ok(lib().psx_chunk_adam_step_unpack(ctx, chunks, nc, C.byref(hyper), flags, t, slots, n, chunk_elems, _stream(stream)))


def psx_chunk_adam_step_noalloc(chunks, hyper, flags=0, flag_out_dev=None, stream=None, n_chunks=None):
    n = len(chunks) if n_chunks is None else n_chunks
    _ok(lib().psx_chunk_adam_step_noalloc(chunks, n, C.byref(hyper), flags, _addr(flag_out_dev), _stream(stream)))


SCALAR_NAMES = ("step_size", "c2", "inv_scale", "beta1", "beta2", "omb1", "omb2", "eps", "wd", "decay")


def psx_adam_step_scalars(hyper):
    """-> dict of the ten fp32 scalars (as Python floats holding exact fp32 values)."""
    out = (C.c_float * 10)()
    _ok(lib().psx_adam_step_scalars(C.byref(hyper), out))
    return dict(zip(SCALAR_NAMES, out))


def psx_step_state_init(ctx, hyper, scaler, stream=None):
    _ok(lib().psx_step_state_init(ctx, C.byref(hyper), C.byref(scaler), _stream(stream)))


def psx_step_state_advance(ctx, flags=0, stream=None):
    _ok(lib().psx_step_state_advance(ctx, flags, _stream(stream)))


def psx_step_state_read(ctx, stream=None):
    """-> (psx_scaler, flag of the step closed last, steps skipped so far); synchronises."""
    s, flag, skipped = psx_scaler(), C.c_uint32(0), C.c_uint64(0)
    _ok(lib().psx_step_state_read(ctx, C.byref(s), C.byref(flag), C.byref(skipped), _stream(stream)))
    return s, flag.value, skipped.value


def make_scaler(scale=65536.0, growth_interval=2000):
    return psx_scaler(scale, growth_interval, 0, 0, 1)


def psx_loss_scale_update(scaler, overflow):
    _ok(lib().psx_loss_scale_update(C.byref(scaler), int(bool(overflow))))


def psx_ctx_set_tuning(ctx, key, value):
    _ok(lib().psx_ctx_set_tuning(ctx, key, value))


def psx_ctx_set_profiling(ctx, on):
    _ok(lib().psx_ctx_set_profiling(ctx, int(on)))


def psx_ctx_get_timing(ctx):
    t = psx_timing()
    _ok(lib().psx_ctx_get_timing(ctx, C.byref(t)))
    return t


def psx_copy_bytes(ctx, dst, src, n_bytes, stream=None):
    _ok(lib().psx_copy_bytes(ctx, _addr(dst), _addr(src), n_bytes, _stream(stream)))


def psx_measure_link(ctx, mib=1024, reps=5):
    r = psx_link_rates()
    _ok(lib().psx_measure_link(ctx, mib, reps, C.byref(r)))
    return r


def psx_pinned_alloc(n_bytes):
    """-> integer address of page-locked, device-accessible host memory."""
    out = C.c_void_p(0)
    _ok(lib().psx_pinned_alloc(n_bytes, C.byref(out)))
    return out.value


def psx_pinned_free(addr):
    _ok(lib().psx_pinned_free(C.c_void_p(addr)))


class PinnedF32:
    """n float32 elements of pinned host memory from psx_pinned_alloc, with a numpy view.
    `data_ptr()` makes it usable wherever the binding takes a tensor."""

    def __init__(self, n, fill=0.0):
        import numpy as np
        self.n = int(n)
        self.addr = psx_pinned_alloc(max(self.n, 1) * 4)
        self.np = np.ctypeslib.as_array((C.c_float * max(self.n, 1)).from_address(self.addr))[:self.n]
        self.np[...] = fill

    def data_ptr(self):
        return self.addr

    def free(self):
        if self.addr:
            self.np = None
            psx_pinned_free(self.addr)
            self.addr = 0


def psx_plan_residency(used, chunk_elems, hbm_budget_bytes):
    """-> (loc list of PSX_LOC_*, host_elems)."""
    n = len(used)
    u = (C.c_uint64 * max(n, 1))(*used)
    loc = (C.c_uint8 * max(n, 1))()
    host = C.c_uint64(0)
    _ok(lib().psx_plan_residency(u, n, chunk_elems, hbm_budget_bytes, loc, C.byref(host)))
    return list(loc)[:n], host.value


def psx_chunk_size_search(numel, lo, hi, step, flags=0, max_model_data_bytes=0):
    """-> (best chunk_elems, utilisation, n_chunks)."""
    n = len(numel)
    arr = (C.c_uint64 * max(n, 1))(*numel)
    best, util, nch = C.c_uint64(0), C.c_double(0), C.c_size_t(0)
    _ok(lib().psx_chunk_size_search(arr, n, lo, hi, step, flags, max_model_data_bytes, C.byref(best),
                                    C.byref(util), C.byref(nch)))
    return best.value, util.value, nch.value
