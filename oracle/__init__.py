"""ctypes loader for the scalar CPU oracle (oracle/psx_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
benchmark's cpu_baseline leg import this package.  It marshals numpy arrays
into the plain C routines and holds no arithmetic of its own.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "psx_oracle.c")
_LIB = os.path.join(_HERE, "libpsx_oracle.so")
# the mutation test points this at deliberately broken builds to prove that the pins notice them
_LIB_OVERRIDE = os.environ.get("PSX_ORACLE_LIB")

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c11", "-Wall"]


def build(force=True):
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Slot(C.Structure):
    _fields_ = [("chunk", C.c_uint32), ("reserved", C.c_uint32),
                ("offset", C.c_uint64), ("numel", C.c_uint64)]


class AdamHyper(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("loss_scale", C.c_double),
                ("step", C.c_uint64), ("adamw_mode", C.c_uint32), ("reserved", C.c_uint32)]


class AdamScalars(C.Structure):
    _fields_ = [(k, C.c_float) for k in ("step_size", "c2", "inv_scale", "beta1", "beta2",
                                         "omb1", "omb2", "eps", "wd", "decay")]


class Scaler(C.Structure):
    _fields_ = [("scale", C.c_float), ("growth_interval", C.c_uint32),
                ("good_steps", C.c_uint32), ("reserved", C.c_uint32),
                ("step", C.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if _LIB_OVERRIDE:
            L = C.CDLL(_LIB_OVERRIDE)
        else:
            build(force=False)
            L = C.CDLL(_LIB)
        L.orc_f16_to_f32.restype = C.c_float
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_f16_to_f32_array.restype = None
        L.orc_f16_to_f32_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_f32_to_f16_array.restype = None
        L.orc_f32_to_f16_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_chunk_layout.restype = C.c_int
        L.orc_chunk_layout.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int,
                                       C.c_void_p, C.c_void_p, C.c_uint64,
                                       C.POINTER(C.c_uint64)]
        L.orc_pack.restype = None
        L.orc_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                               C.c_uint64, C.c_uint64]
        L.orc_unpack.restype = None
        L.orc_unpack.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                                 C.c_uint64, C.c_uint64]
        L.orc_overflow_check.restype = C.c_uint32
        L.orc_overflow_check.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.orc_adam_prepare.restype = None
        L.orc_adam_prepare.argtypes = [C.POINTER(AdamHyper), C.POINTER(AdamScalars)]
        L.orc_adam_chunk.restype = None
        L.orc_adam_chunk.argtypes = [C.c_void_p] * 5 + [C.c_uint64, C.POINTER(AdamHyper)]
        L.orc_recast_chunk.restype = None
        L.orc_recast_chunk.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_chunk_adam_step.restype = C.c_uint32
        L.orc_chunk_adam_step.argtypes = [C.c_void_p] * 6 + [C.c_uint64, C.POINTER(AdamHyper)]
        L.orc_min_link_bytes.restype = C.c_uint64
        L.orc_min_link_bytes.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
        L.orc_scaler_update.restype = None
        L.orc_scaler_update.argtypes = [C.POINTER(Scaler), C.c_uint32]
        _lib = L
    return _lib


# ---------------------------------------------------------------- marshalling

def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _ptr_array(arrays):
    return (C.c_void_p * len(arrays))(*[None if a is None else a.ctypes.data for a in arrays])


def _check(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    return a


def f16_to_f32(h_bits):
    h = _check(np.ascontiguousarray(h_bits), np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().orc_f16_to_f32_array(_ptr(h), _ptr(out), h.size)
    return out


def f32_to_f16(f):
    f = _check(np.ascontiguousarray(f), np.float32)
    out = np.empty(f.shape, np.uint16)
    lib().orc_f32_to_f16_array(_ptr(f), _ptr(out), f.size)
    return out


def chunk_layout(numel, chunk_elems, strict=False):
    """Return (slots as a numpy structured array, used[n_chunks]) or raise ValueError."""
    numel = np.ascontiguousarray(numel, dtype=np.uint64)
    n = numel.size
    nch = C.c_uint64(0)
    rc = lib().orc_chunk_layout(_ptr(numel), n, chunk_elems, int(strict), None, None, 0,
                                C.byref(nch))
    if rc != 0:
        raise ValueError(f"orc_chunk_layout rc={rc}")
    slots = (Slot * max(n, 1))()
    used = np.zeros(nch.value, np.uint64)
    rc = lib().orc_chunk_layout(_ptr(numel), n, chunk_elems, int(strict), slots, _ptr(used),
                                used.size, C.byref(nch))
    if rc != 0:
        raise ValueError(f"orc_chunk_layout rc={rc}")
    return slots, used


def slots_as_tuples(slots, n):
    return [(slots[i].chunk, slots[i].offset, slots[i].numel) for i in range(n)]


def pack(tensors, slots, chunks, chunk_elems):
    """tensors: list of 1-D numpy arrays; chunks: list of 1-D numpy arrays (same dtype); a chunk may
    be None (not materialised: its elements are skipped)."""
    es = next(c for c in chunks if c is not None).dtype.itemsize
    for t in tensors:
        assert t.dtype.itemsize == es and t.flags.c_contiguous
    for c in chunks:
        assert c is None or (c.size == chunk_elems and c.flags.c_contiguous)
    lib().orc_pack(_ptr_array(tensors), slots, len(tensors), _ptr_array(chunks), chunk_elems, es)


def unpack(tensors, slots, chunks, chunk_elems):
    es = next(c for c in chunks if c is not None).dtype.itemsize
    for t in tensors:
        assert t.dtype.itemsize == es and t.flags.c_contiguous
    lib().orc_unpack(_ptr_array(tensors), slots, len(tensors), _ptr_array(chunks), chunk_elems, es)


def overflow_check(g16_chunks, used):
    """g16_chunks: list of uint16 arrays (fp16 bit patterns). Returns (flag, per_chunk)."""
    for c in g16_chunks:
        _check(c, np.uint16)
    used = np.ascontiguousarray(used, dtype=np.uint64)
    per = np.zeros(len(g16_chunks), np.uint32)
    flag = lib().orc_overflow_check(_ptr_array(g16_chunks), _ptr(used), len(g16_chunks), _ptr(per))
    return int(flag), per


def hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, adamw_mode=0, step=1,
          loss_scale=1.0):
    return AdamHyper(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay),
                     float(loss_scale), int(step), int(adamw_mode), 0)


def adam_prepare(h):
    s = AdamScalars()
    lib().orc_adam_prepare(C.byref(h), C.byref(s))
    return s


def adam_chunk(g16, p16, p32, m, v, used, h):
    """In-place update of one chunk's first `used` elements. g16/p16: uint16 bit patterns."""
    _check(g16, np.uint16); _check(p16, np.uint16)
    _check(p32, np.float32); _check(m, np.float32); _check(v, np.float32)
    assert min(g16.size, p16.size, p32.size, m.size, v.size) >= used
    lib().orc_adam_chunk(_ptr(g16), _ptr(p16), _ptr(p32), _ptr(m), _ptr(v), int(used), C.byref(h))


def recast_chunk(p16, p32, used):
    _check(p16, np.uint16); _check(p32, np.float32)
    lib().orc_recast_chunk(_ptr(p16), _ptr(p32), int(used))


def chunk_adam_step(g16, p16, p32, m, v, used, h):
    """Whole step over chunk lists (lists of numpy arrays); returns the overflow flag."""
    used = np.ascontiguousarray(used, dtype=np.uint64)
    n = len(p32)
    # keep g16[c] is p16[c] aliasing visible to the C side through equal pointers
    return int(lib().orc_chunk_adam_step(_ptr_array(g16), _ptr_array(p16), _ptr_array(p32),
                                         _ptr_array(m), _ptr_array(v), _ptr(used), n,
                                         C.byref(h)))


def scaler(scale=65536.0, growth_interval=2000):
    return Scaler(scale, growth_interval, 0, 0, 1)


def scaler_update(s, overflow):
    lib().orc_scaler_update(C.byref(s), int(bool(overflow)))


def min_link_bytes(used, budgets_in_chunks, start_resident):
    """Brute-force least link bytes of the ADAM scan over len(budgets) steps (tiny cases only)."""
    used = np.ascontiguousarray(used, dtype=np.uint64)
    b = np.ascontiguousarray(budgets_in_chunks, dtype=np.uint64)
    st = np.ascontiguousarray(start_resident, dtype=np.uint8)
    assert used.size * b.size <= 24
    return int(lib().orc_min_link_bytes(_ptr(used), used.size, _ptr(b), b.size, _ptr(st)))
