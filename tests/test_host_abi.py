"""CPU-side tests of the C-ABI library: it loads, exports every symbol the
header declares, and its host-only entry points (layout, loss scaler, argument
validation) agree with the oracle.  No GPU work is issued here."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

from paper_2108_05818_amd import psx
from paper_2108_05818_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "psx.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(psx_[a-z0-9_]+)\s*\(", header))
    assert declared == set(psx.EXPORTS)
    L = psx.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_header_is_plain_c_and_binding_structs_match_it(tmp_path):
    """include/psx.h must compile as strict C99 on its own, and every struct of the Python binding must have
    the size and field offsets the C compiler gives it (a marshalling mismatch would corrupt arguments
    silently).  Constants the binding repeats are compared as well."""
    import subprocess
    structs = [psx.psx_slot, psx.psx_ctx_config, psx.psx_adam_hyper, psx.psx_chunk, psx.psx_scaler,
               psx.psx_timing, psx.psx_link_rates]
    consts = [n for n in dir(psx) if n.startswith("PSX_") and isinstance(getattr(psx, n), int)]
    header = open(os.path.join(ROOT, "include", "psx.h")).read()
    consts = [n for n in consts if re.search(r"#define\s+%s\b" % n, header)]
    assert len(consts) > 25
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "psx.h"', 'int main(void) {']
    for st in structs:
        n = st.__name__
        lines.append(f'printf("{n} %zu\\n", sizeof({n}));')
        for f, _ in st._fields_:
            lines.append(f'printf("{n}.{f} %zu\\n", offsetof({n}, {f}));')
    for n in consts:
        lines.append(f'printf("{n} %lld\\n", (long long)({n}));')
    lines.append('return 0; }')
    src = tmp_path / "abi.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st in structs:
        n = st.__name__
        assert int(got[n]) == C.sizeof(st), n
        for f, _ in st._fields_:
            assert int(got[f"{n}.{f}"]) == getattr(st, f).offset, f"{n}.{f}"
    for n in consts:
        assert int(got[n]) == getattr(psx, n), n


def _same_layout(orc, numel, C_, flags=0):
    o_slots, o_used = orc.chunk_layout(numel, C_, strict=bool(flags & psx.PSX_LAYOUT_STRICT))
    slots, used = psx.psx_chunk_layout(numel, C_, flags)
    assert used == [int(u) for u in o_used]
    for i in range(len(numel)):
        assert (slots[i].chunk, slots[i].offset, slots[i].numel) == \
               (o_slots[i].chunk, o_slots[i].offset, o_slots[i].numel), (numel, C_, i)


def test_layout_matches_oracle_exhaustive_small(orc):
    for n in range(0, 5):
        for numel in itertools.product([0, 1, 2, 3, 5, 8, 13], repeat=n):
            for C_ in (1, 2, 3, 4, 5, 8, 16):
                _same_layout(orc, list(numel), C_)


def test_layout_matches_oracle_random_and_configs(orc):
    rng = np.random.default_rng(3)
    for _ in range(300):
        n = int(rng.integers(1, 60))
        C_ = int(rng.integers(1, 100))
        _same_layout(orc, [int(x) for x in rng.integers(0, 3 * C_, size=n)], C_)
    for w in (W.config1_tiny(), W.config2_gpt1b(), W.config3_ragged(), W.config4_gpt12b(), W.config5_gpt20b()):
        _same_layout(orc, w.numel, w.chunk_elems)
    w = W.config1_tiny()
    _same_layout(orc, w.numel, w.chunk_elems, psx.PSX_LAYOUT_STRICT)


def test_layout_errors():
    with pytest.raises(psx.PsxError) as e:
        psx.psx_chunk_layout([4, 9, 2], 8, psx.PSX_LAYOUT_STRICT)
    assert e.value.code == psx.PSX_ETOOLARGE and "tensor 1" in str(e.value)
    with pytest.raises(psx.PsxError) as e:
        psx.psx_chunk_layout([1], 0)
    assert e.value.code == psx.PSX_EINVAL
    # used[] too short
    L = psx.lib()
    numel = (C.c_uint64 * 3)(8, 8, 8)
    used = (C.c_uint64 * 2)(7, 7)
    nch = C.c_size_t(0)
    assert L.psx_chunk_layout(numel, 3, 8, 0, None, used, 2, C.byref(nch)) == psx.PSX_ECAP
    assert list(used) == [7, 7]                      # nothing written on error
    assert L.psx_chunk_layout(numel, 3, 8, 0x80, None, None, 0, C.byref(nch)) == psx.PSX_EINVAL
    assert L.psx_chunk_layout(None, 3, 8, 0, None, None, 0, C.byref(nch)) == psx.PSX_EINVAL


def test_scaler_matches_oracle(orc):
    rng = np.random.default_rng(12)
    for gi in (1, 2, 3, 50):
        a = psx.make_scaler(65536.0, gi)
        b = orc.scaler(65536.0, gi)
        for ov in rng.random(400) < 0.15:
            psx.psx_loss_scale_update(a, ov)
            orc.scaler_update(b, ov)
            assert (a.scale, a.good_steps, a.step) == (b.scale, b.good_steps, b.step)


def test_null_arguments_are_errors_not_crashes():
    L = psx.lib()
    assert L.psx_loss_scale_update(None, 0) == psx.PSX_EINVAL
    assert L.psx_ctx_create(None, None) == psx.PSX_EINVAL
    assert L.psx_ctx_destroy(None) == psx.PSX_OK
    assert L.psx_pack(None, 1, None, None, 0, None, 0, 8, 0, None) == psx.PSX_EINVAL
    assert L.psx_overflow_check(None, None, None, 0, None, None, None) == psx.PSX_EINVAL
    assert L.psx_chunk_adam_step(None, None, 0, None, 0, None) == psx.PSX_EINVAL
    assert b"ctx is NULL" in L.psx_last_error()


def test_noalloc_step_validates_before_it_touches_the_gpu():
    """Size and flag errors of psx_chunk_adam_step_noalloc are found on the host, before any HIP call."""
    L = psx.lib()
    h = psx.make_hyper()
    assert L.psx_chunk_adam_step_noalloc(None, 0, None, 0, None, None) == psx.PSX_EINVAL
    assert L.psx_chunk_adam_step_noalloc(None, 1, C.byref(h), 0, None, None) == psx.PSX_EINVAL
    spec = dict(g16=1 << 20, p16=1 << 20, p32=1 << 21, m=1 << 22, v=1 << 23, used=8)
    many = psx.make_chunks([spec] * (psx.PSX_NOALLOC_MAX_CHUNKS + 1))
    assert L.psx_chunk_adam_step_noalloc(many, len(many), C.byref(h), 0, None, None) == psx.PSX_ECAP
    one = psx.make_chunks([spec])
    assert L.psx_chunk_adam_step_noalloc(one, 1, C.byref(h), psx.PSX_STEP_USE_FLAG, None, None) == psx.PSX_EINVAL
    assert L.psx_chunk_adam_step_noalloc(one, 1, C.byref(h), 0, 1 << 24, None) == psx.PSX_EINVAL   # flag_out needs the check
    odd = psx.make_chunks([dict(spec, m=(1 << 22) + 4)])
    assert L.psx_chunk_adam_step_noalloc(odd, 1, C.byref(h), 0, None, None) == psx.PSX_EALIGN
    bad = psx.make_hyper(step=0)
    assert L.psx_chunk_adam_step_noalloc(one, 1, C.byref(bad), 0, None, None) == psx.PSX_EINVAL


def test_step_scalars_agree_with_the_oracle_over_many_steps(orc):
    """Library and oracle both define beta^t as the product of t factors in double, each in code of its
    own (the library continues the product of its last call, the oracle starts from 1 every time).  All
    ten scalars must be the same fp32 numbers at every step: every t up to 20000, then every 97th up to
    10^5, for several betas; steps asked for out of order; a power that has underflowed to zero; and the
    one step found where libm's pow would have given another c2 (beta2 = 0.999999, t = 12314)."""
    def same(hp, t):
        mine = psx.psx_adam_step_scalars(psx.make_hyper(step=t, **hp))
        ref = orc.adam_prepare(orc.hyper(step=t, **hp))
        for name in psx.SCALAR_NAMES:
            assert mine[name] == getattr(ref, name), (hp, t, name)
        return mine
    cases = [dict(lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.01, loss_scale=65536.0),
             dict(lr=3e-4, beta1=0.95, beta2=0.98, weight_decay=0.1, adamw_mode=1, loss_scale=1024.0),
             dict(lr=1e-2, beta1=0.8, beta2=0.9999, eps=1e-6, loss_scale=1.0),
             dict(lr=5e-4, beta1=0.0, beta2=0.5, loss_scale=3.0)]
    for i, hp in enumerate(cases):
        steps = list(range(1, 20001 if i == 0 else 2001)) + list(range(20001, 100001, 97 if i == 0 else 4999))
        for t in steps:
            same(hp, t)
    near_one = dict(lr=1e-3, beta1=0.9, beta2=0.999999, loss_scale=1.0)
    import math
    for t in (12313, 12314, 12315, 7, 12314, 1, 250000, 12314):          # forwards, back, and again
        got = same(near_one, t)
    by_pow = np.float32(1.0 / math.sqrt(1.0 - math.pow(0.999999, 12314)))
    assert got["c2"] != by_pow and abs(float(got["c2"]) - float(by_pow)) <= float(np.spacing(by_pow))
    for t in (3_000_000, 2_999_999, 3_000_001):                           # 0.999^t is zero in double by then
        got = same(cases[0], t)
        assert got["c2"] == 1.0 and got["step_size"] == np.float32(1e-3)
    with pytest.raises(psx.PsxError):
        psx.psx_adam_step_scalars(psx.make_hyper(step=0))
    with pytest.raises(psx.PsxError):
        psx.psx_adam_step_scalars(psx.make_hyper(beta2=1.0))


def test_bench_refuses_more_than_one_gpu():
    """The path has no collectives and every box has one GPU: `bench.py --gpus N` with N > 1 says so and exits."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
