"""The C ABI used from a plain C program (tests/c_abi_driver.c: no Python, no PyTorch, hipMalloc'ed
memory, the system HIP runtime) against the oracle.  The program is built by `__graft_entry__.build()`
next to its source; this test writes a seeded case to a file, runs the program as a child process,
and compares every byte it wrote with what the oracle computes from the same input."""
import os
import struct
import subprocess

import numpy as np
import pytest

from paper_2108_05818_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))
DRIVER = os.path.join(HERE, "c_abi_driver")
MAGIC = 0x7073785f63616269

pytestmark = pytest.mark.gpu


def run_case(orc, tmp_path, numel, C, steps, hp, scale0, growth, bad_steps, host_from=1 << 40):
    assert os.path.exists(DRIVER), f"{DRIVER} is missing: build it with `python __graft_entry__.py`"
    n, N = len(numel), int(sum(numel))
    params = [W.params_np(s, 8100 + i) for i, s in enumerate(numel)]
    # the loss scale a step will run with is known in advance only from the oracle's own scaler: run it first
    sc = orc.scaler(scale0, growth)
    slots, used = orc.chunk_layout(numel, C)
    nch = used.size
    lists = {k: [np.zeros(C, np.uint16 if k in ("g16", "p16") else np.float32) for _ in range(nch)] for k in ("g16", "p16", "p32", "m", "v")}
    orc.pack(params, slots, lists["p32"], C)
    grads_all, trace = [], []
    for t in range(steps):
        grads = [W.grads_f16_np(s, 9100 + 100 * t + i, float(sc.scale)) for i, s in enumerate(numel)]
        if t in bad_steps:
            big = max(range(n), key=lambda i: numel[i])
            grads[big][numel[big] // 2] = 0x7C00 if t % 2 else 0xFE01          # +inf or a NaN
        grads_all.append(grads)
        orc.pack(grads, slots, lists["g16"], C)
        h = orc.hyper(step=sc.step, loss_scale=sc.scale, **hp)
        flag = orc.chunk_adam_step(lists["g16"], lists["p16"], lists["p32"], lists["m"], lists["v"], used, h)
        orc.scaler_update(sc, flag)
        trace.append((flag, float(sc.scale)))
    p16_t = [np.zeros(s, np.uint16) for s in numel]
    orc.unpack(p16_t, slots, lists["p16"], C)

    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        f.write(struct.pack("<7Q", MAGIC, n, C, steps, int(hp.get("adamw_mode", 0)), growth, host_from))
        f.write(struct.pack("<6d", hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"], scale0))
        f.write(np.asarray(numel, np.uint64).tobytes())
        for p in params:
            f.write(p.tobytes())
        for grads in grads_all:
            for g in grads:
                f.write(g.tobytes())
    r = subprocess.run([DRIVER, str(fin), str(fout)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    raw = open(fout, "rb").read()
    pos = 0

    def take(dtype, count):
        nonlocal pos
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=pos)
        pos += a.nbytes
        return a
    assert int(take(np.uint64, 1)[0]) == nch
    assert np.array_equal(take(np.uint64, nch), used)
    for t in range(steps):
        flag = int(take(np.uint32, 1)[0])
        scale = float(take(np.float32, 1)[0])
        assert (flag, scale) == trace[t], (t, flag, scale, trace[t])
    for k in range(nch):
        u = int(used[k])
        for name in ("p32", "m", "v"):
            assert take(np.float32, u).tobytes() == lists[name][k][:u].tobytes(), (k, name)
        assert np.array_equal(take(np.uint16, u), lists["p16"][k][:u]), (k, "p16")
    got = take(np.uint16, N)
    assert np.array_equal(got, np.concatenate(p16_t) if n else got)
    assert pos == len(raw)
    return trace


def test_plain_c_program_matches_the_oracle(orc, tmp_path):
    """Ragged tensors (single elements, one larger than a chunk, sizes that leave every alignment), chunks of
    4104 elements, 7 steps of which two overflow, growth interval 2: flags, loss scale, fp32 states, fp16
    parameter chunks and the unpacked fp16 tensors, bit for bit."""
    numel = [1, 4000, 7, 9001, 333, 1, 2049, 4104, 15, 640]
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, adamw_mode=0)
    trace = run_case(orc, tmp_path, numel, 4104, 7, hp, 1024.0, 2, bad_steps={2, 5})
    assert [f for f, _ in trace] == [0, 0, 1, 0, 0, 1, 0]
    assert {s for _, s in trace} == {1024.0, 2048.0}


def test_plain_c_program_with_host_resident_chunks(orc, tmp_path):
    """The same list with the fp32 states of chunks 2.. in pinned host memory (psx_pinned_alloc), updated over
    the link by the kernel under the system HIP runtime; one overflow."""
    numel = [1, 4000, 7, 9001, 333, 1, 2049, 4104, 15, 640]
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, adamw_mode=0)
    trace = run_case(orc, tmp_path, numel, 4104, 5, hp, 1024.0, 2, bad_steps={1}, host_from=2)
    assert [f for f, _ in trace] == [0, 1, 0, 0, 0]


def test_plain_c_program_decoupled_decay_one_chunk(orc, tmp_path):
    hp = dict(lr=3e-4, beta1=0.8, beta2=0.99, eps=1e-6, weight_decay=0.1, adamw_mode=1)
    run_case(orc, tmp_path, [70000, 12345, 3], 1 << 17, 3, hp, 65536.0, 2000, bad_steps=set())
