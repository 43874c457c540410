"""GPU parity: the HIP path, called through the C ABI, against the scalar CPU
oracle on the same seeded inputs.  Bit-exact for layout, pack/unpack, flags and
the fp16 re-cast; p/m/v within 2 ulp (0 expected: same operations, same order,
IEEE-correct on both sides).  The oracle runs free on its own copy of the
seeded inputs: nothing the HIP path produced is ever fed to it."""
import numpy as np
import pytest
import torch

from paper_2108_05818_amd import psx
from paper_2108_05818_amd import workloads as W

from gpu_util import DEV, SENT16, SENT32, ChunkLists, bits16, bits32, f32, from_bits16, sent16, sent32

pytestmark = pytest.mark.gpu

H, G = psx.PSX_LOC_HOST, psx.PSX_LOC_HBM


@pytest.fixture(scope="module")
def ctx():
    c = psx.psx_ctx_create(max_chunks=512, max_tensors=8192, staging_tile_elems=4096, staging_slots=3)
    yield c
    psx.psx_ctx_destroy(c)


def fill_state(cl, seed, loss_scale, zero_mv=True):
    for k in range(cl.n):
        u = cl.used[k]
        if u == 0:
            continue
        cl.set("p32", k, W.params_np(u, seed + 10 * k))
        if zero_mv:
            cl.set("m", k, np.zeros(u, np.float32))
            cl.set("v", k, np.zeros(u, np.float32))
        else:
            cl.set("m", k, W.params_np(u, seed + 10 * k + 1) * np.float32(0.05))
            cl.set("v", k, np.abs(W.params_np(u, seed + 10 * k + 2)) * np.float32(1e-4))
        cl.set("g16", k, W.grads_f16_np(u, seed + 10 * k + 3, loss_scale))


def check_recast_of_own_params(orc, cl):
    """p16 must be exactly the fp16 (round to nearest even) of the GPU's own fp32 params."""
    for k in range(cl.n):
        u = cl.used[k]
        assert np.array_equal(bits16(cl.p16[k])[:u], orc.f32_to_f16(f32(cl.p32[k])[:u])), f"chunk {k}"


# ---------------------------------------------------------------------------------- config 1, end to end

@pytest.mark.parametrize("alias", [False, True])
def test_config1_tiny_gpt_ten_steps(orc, ctx, alias):
    w = W.config1_tiny()
    slots, used = psx.psx_chunk_layout(w.numel, w.chunk_elems)
    o_slots, o_used = orc.chunk_layout(w.numel, w.chunk_elems)
    assert used == [int(u) for u in o_used]
    nch, Cn = len(used), w.chunk_elems
    cl = ChunkLists(used, Cn, alias=alias)

    # params: fp32 tensors packed into the p32 list on both sides; m = v = 0
    p_np = [W.params_np(s, w.seed + i) for i, s in enumerate(w.numel)]
    psx.psx_pack(ctx, psx.PSX_F32, [torch.from_numpy(a).to(DEV) for a in p_np], slots, cl.p32, Cn)
    orc.pack(p_np, o_slots, cl.np["p32"], Cn)
    for k in range(nch):
        cl.set("m", k, np.zeros(used[k], np.float32))
        cl.set("v", k, np.zeros(used[k], np.float32))
    cl.compare("after param pack")

    scaler = psx.make_scaler(w.loss_scale, w.growth_interval)
    o_scaler = orc.scaler(w.loss_scale, w.growth_interval)
    worst = 0.0
    for step in range(w.steps):
        g_np = [W.grads_f16_np(s, w.seed + 1000 * (step + 1) + i, scaler.scale) for i, s in enumerate(w.numel)]
        psx.psx_pack(ctx, psx.PSX_F16, [from_bits16(a) for a in g_np], slots, cl.g16, Cn)
        orc.pack(g_np, o_slots, cl.np["g16"], Cn)
        for k in range(nch):
            assert bits16(cl.g16[k]).tobytes() == cl.np["g16"][k].tobytes()
        flag, per = psx.psx_overflow_check(ctx, cl.g16, used)
        o_flag, o_per = orc.overflow_check(cl.np["g16"], np.array(used, np.uint64))
        assert (flag, per) == (o_flag, list(o_per)) == (0, [0] * nch)
        hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                  adamw_mode=w.adamw_mode, step=scaler.step, loss_scale=scaler.scale)
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(**hp), psx.PSX_STEP_USE_FLAG)
        torch.cuda.synchronize()
        assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
        worst = max(worst, cl.compare(f"step {step}"))
        check_recast_of_own_params(orc, cl)
        psx.psx_loss_scale_update(scaler, flag)
        orc.scaler_update(o_scaler, o_flag)
        assert (scaler.scale, scaler.step) == (o_scaler.scale, o_scaler.step)
    print(f"config1 alias={alias}: worst error over {w.steps} free-running steps: {worst} ulp")
    # unpack the fp16 params back into tensors
    out = [torch.zeros(s, dtype=torch.float16, device=DEV) for s in w.numel]
    psx.psx_unpack(ctx, psx.PSX_F16, out, slots, cl.p16, Cn)
    o_out = [np.zeros(s, np.uint16) for s in w.numel]
    orc.unpack(o_out, o_slots, cl.np["p16"], Cn)
    torch.cuda.synchronize()
    for a, b in zip(out, o_out):
        assert bits16(a).tobytes() == b.tobytes()


# ---------------------------------------------------------------------------------- pack / unpack

COPY_SHAPES = [(64, 0, 0, 1), (256, 1, 0, 1), (64, 4, 0, 0), (256, 4, 2, 1), (64, 1, 1, 0)]
COPY_KEYS = [psx.PSX_TUNE_COPY_THREADS, psx.PSX_TUNE_COPY_UNROLL, psx.PSX_TUNE_COPY_BLOCKS_PER_CU, psx.PSX_TUNE_NONTEMPORAL]


class copy_shape:
    """Select a pack/unpack launch shape (threads, vectors per thread, persistent workgroups per CU,
    non-temporal) on the shared context for the length of a with-block; COPY_SHAPES[0] is the default."""

    def __init__(self, ctx, shape):
        self.ctx, self.shape = ctx, shape

    def __enter__(self):
        for key, val in zip(COPY_KEYS, self.shape):
            psx.psx_ctx_set_tuning(self.ctx, key, val)

    def __exit__(self, *exc):
        for key, val in zip(COPY_KEYS, COPY_SHAPES[0]):
            psx.psx_ctx_set_tuning(self.ctx, key, val)


@pytest.mark.parametrize("shape", COPY_SHAPES)
@pytest.mark.parametrize("dtype", [psx.PSX_F16, psx.PSX_F32])
def test_pack_unpack_ragged_unaligned(orc, ctx, dtype, shape):
    with copy_shape(ctx, shape):
        _pack_unpack_ragged_unaligned(orc, ctx, dtype)


def _pack_unpack_ragged_unaligned(orc, ctx, dtype):
    rng = np.random.default_rng(77)
    Cn = 20000
    numel = [1, 3, 0, 7, 8, 9, 8191, 8193, 1, 16384, 2, 45001, 5, 19999, 20000, 1, 61234, 33, 4095, 1, 1, 12345, 8192]
    numel += [int(x) for x in rng.integers(0, 3000, size=150)]
    npd, ipd, sent = (np.uint16, np.int16, SENT16) if dtype == psx.PSX_F16 else (np.uint32, np.int32, SENT32)
    slots, used = psx.psx_chunk_layout(numel, Cn)
    o_slots, o_used = orc.chunk_layout(numel, Cn)
    nch = len(used)
    # tensors carved at odd element offsets out of one buffer, so sources are misaligned in every way
    gaps = [int(x) for x in rng.integers(0, 3, size=len(numel))]
    total = sum(numel) + sum(gaps) + 16
    big = rng.integers(0, np.iinfo(npd).max, size=total, dtype=np.uint64).astype(npd)
    big_t = torch.from_numpy(big.view(ipd)).to(DEV)
    t_np, t_dev, pos = [], [], 1
    for s, gap in zip(numel, gaps):
        t_np.append(np.ascontiguousarray(big[pos:pos + s]))
        t_dev.append(big_t[pos:pos + s])
        pos += s + gap
    chunks = [torch.from_numpy(np.full(Cn, sent, npd).view(ipd)).to(DEV) for _ in range(nch)]
    o_chunks = [np.full(Cn, sent, npd) for _ in range(nch)]
    psx.psx_pack(ctx, dtype, t_dev, slots, chunks, Cn)
    orc.pack(t_np, o_slots, o_chunks, Cn)
    torch.cuda.synchronize()
    for k in range(nch):
        assert chunks[k].cpu().numpy().view(npd).tobytes() == o_chunks[k].tobytes(), f"chunk {k}"
    # unpack into fresh, equally misaligned tensors; nothing outside them may be written
    out_big = torch.zeros_like(big_t)
    outs, pos, mask = [], 1, np.ones(total, bool)
    for s, gap in zip(numel, gaps):
        outs.append(out_big[pos:pos + s])
        mask[pos:pos + s] = False
        pos += s + gap
    psx.psx_unpack(ctx, dtype, outs, slots, chunks, Cn)
    torch.cuda.synchronize()
    for a, b in zip(outs, t_np):
        assert a.cpu().numpy().view(npd).tobytes() == b.tobytes()
    assert not out_big.cpu().numpy()[mask].any()


@pytest.mark.parametrize("shape", COPY_SHAPES)
def test_pack_with_fused_overflow_check(orc, ctx, shape):
    with copy_shape(ctx, shape):
        _pack_with_fused_overflow_check(orc, ctx)


def _pack_with_fused_overflow_check(orc, ctx):
    Cn = 30000
    numel = [1, 17, 29999, 30000, 5, 70001, 12, 8192, 1]
    slots, used = psx.psx_chunk_layout(numel, Cn)
    o_slots, _ = orc.chunk_layout(numel, Cn)
    nch = len(used)
    base = [W.grads_f16_np(s, 500 + i, 1024.0) for i, s in enumerate(numel)]
    cases = [None, (0, 0), (1, 16), (2, 29998), (5, 70000), (5, 31000), (8, 0), (6, 11)]
    for case in cases:
        g_np = [a.copy() for a in base]
        if case is not None:
            g_np[case[0]][case[1]] = 0x7C00 if case[1] % 2 == 0 else 0xFE01
        chunks = [from_bits16(np.full(Cn, 0x7C00, np.uint16)) for _ in range(nch)]     # inf in the padding
        o_chunks = [np.full(Cn, 0x7C00, np.uint16) for _ in range(nch)]
        psx.psx_overflow_reset(ctx)
        psx.psx_pack(ctx, psx.PSX_F16, [from_bits16(a) for a in g_np], slots, chunks, Cn,
                     flags=psx.PSX_PACK_CHECK_OVERFLOW)
        flag, per = psx.psx_overflow_read(ctx, nch)
        orc.pack(g_np, o_slots, o_chunks, Cn)
        o_flag, o_per = orc.overflow_check(o_chunks, np.array(used, np.uint64))
        assert (flag, per) == (o_flag, list(o_per)), case
        assert flag == (0 if case is None else 1)
        for k in range(nch):
            assert bits16(chunks[k]).tobytes() == o_chunks[k].tobytes()


# ---------------------------------------------------------------------------------- overflow check

def test_overflow_check_positions(orc, ctx):
    Cn = 3 * 8192 + 100
    used = [Cn, 8192, 8193, 1, 0, 16391, 7]
    nch = len(used)
    base = [W.grads_f16_np(Cn, 900 + k, 65536.0) for k in range(nch)]
    for b in base:
        b[(b & 0x7C00) == 0x7C00] = 0x7BFF
    cases = [None]
    for k in range(nch):
        for pos in (0, used[k] - 1, used[k] // 2, used[k], Cn - 1):      # the last two lie in the padding
            if 0 <= pos < Cn:
                cases.append((k, pos))
    specials = W.specials_f16()
    for i, case in enumerate(cases):
        g = [b.copy() for b in base]
        if case is not None:
            g[case[0]][case[1]] = specials[i % len(specials)]
        flag, per = psx.psx_overflow_check(ctx, [from_bits16(a) for a in g], used)
        o_flag, o_per = orc.overflow_check(g, np.array(used, np.uint64))
        assert (flag, per) == (o_flag, list(o_per)), case
        if case is not None:
            assert flag == int(case[1] < used[case[0]])
    # max finite and subnormals never trigger
    g = [np.tile(np.array([0x7BFF, 0xFBFF, 0x0001, 0x83FF], np.uint16), Cn // 4 + 1)[:Cn] for _ in range(nch)]
    flag, per = psx.psx_overflow_check(ctx, [from_bits16(a) for a in g], used)
    assert flag == 0 and not any(per)


# ---------------------------------------------------------------------------------- Adam arithmetic

RAGGED_USED = [1, 3, 4, 5, 1023, 1024, 1025, 2047, 2049, 4096, 4097, 8191, 12289, 0, 20000]


@pytest.mark.parametrize("wd,adamw", [(0.0, 0), (0.01, 0), (0.01, 1)])
@pytest.mark.parametrize("threads,unroll,nt,bpc", [(64, 1, 1, 0), (64, 2, 0, 0), (64, 4, 1, 2), (256, 1, 1, 0),
                                                    (256, 2, 1, 4), (256, 4, 0, 0)])
def test_adam_matches_oracle_over_ragged_chunks(orc, ctx, wd, adamw, threads, unroll, nt, bpc):
    """Every launch shape the tuning knobs can select computes the same bits."""
    defaults = [(psx.PSX_TUNE_ADAM_THREADS, 64), (psx.PSX_TUNE_ADAM_UNROLL, 1), (psx.PSX_TUNE_NONTEMPORAL, 1),
                (psx.PSX_TUNE_ADAM_BLOCKS_PER_CU, 0)]
    for key, val in zip([d[0] for d in defaults], (threads, unroll, nt, bpc)):
        psx.psx_ctx_set_tuning(ctx, key, val)
    try:
        Cn = 20000
        cl = ChunkLists(RAGGED_USED, Cn)
        fill_state(cl, 4000, 65536.0, zero_mv=False)
        # a few special gradients: zeros, fp16 subnormals, largest finite values
        cl.set("g16", 14, np.array([0, 0x8000, 1, 0x8001, 0x03FF, 0x7BFF, 0xFBFF, 0x0400], np.uint16))
        worst = 0.0
        for t in (1, 2, 7):
            hp = dict(lr=1e-3, weight_decay=wd, adamw_mode=adamw, step=t, loss_scale=65536.0)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(**hp))
            torch.cuda.synchronize()
            assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
            worst = max(worst, cl.compare(f"t={t}"))
            check_recast_of_own_params(orc, cl)
        assert worst == 0.0, f"expected bit-exact, got {worst} ulp"
    finally:
        for key, val in defaults:
            psx.psx_ctx_set_tuning(ctx, key, val)


def test_adam_closed_forms_on_gpu(ctx):
    """The closed forms of Kingma & Ba's algorithm, evaluated on the HIP path itself."""
    n = 4096 + 3
    cl = ChunkLists([n], 8192)
    g = np.random.default_rng(1).standard_normal(n).astype(np.float32) * 1e-3
    g16 = (g * 1024).astype(np.float16)
    cl.set("g16", 0, g16.view(np.uint16))
    cl.set("p32", 0, np.full(n, 0.5, np.float32))
    cl.set("m", 0, np.zeros(n, np.float32))
    cl.set("v", 0, np.zeros(n, np.float32))
    psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(lr=1e-3, step=1, loss_scale=1024.0))
    gd = g16.astype(np.float64) / 1024
    want = 0.5 - 1e-3 * gd / (np.abs(gd) + 1e-8)
    assert np.allclose(f32(cl.p32[0])[:n], want, rtol=0, atol=1e-7)
    # zero gradient from zero state: nothing moves
    cl2 = ChunkLists([n], 8192)
    cl2.set("g16", 0, np.zeros(n, np.uint16))
    cl2.set("p32", 0, W.params_np(n, 5))
    cl2.set("m", 0, np.zeros(n, np.float32))
    cl2.set("v", 0, np.zeros(n, np.float32))
    psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl2.specs()), psx.make_hyper(lr=1e-3, step=1, loss_scale=1024.0))
    assert bits32(cl2.p32[0]).tobytes() == cl2.np["p32"][0].view(np.uint32).tobytes()
    assert not f32(cl2.m[0])[:n].any() and not f32(cl2.v[0])[:n].any()


def test_fp16_recast_is_round_to_nearest_even(orc, ctx):
    """Every fp16 tie, its fp32 neighbours, boundaries and subnormals through the kernel's conversion."""
    h = np.arange(0, 0x7C00, dtype=np.uint32).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0
    mid = ((lo + hi) / 2).astype(np.float32)
    vals = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)),
                           lo.astype(np.float32), W.params_np(50000, 6),
                           np.array([0, 65504, 65519.99, 65520, 65536, 1e30, np.inf, 2.0 ** -24, 2.0 ** -25,
                                     2.0 ** -26, 1e-45, 1.17549435e-38, 3.4e38], np.float32)])
    vals = np.concatenate([vals, -vals]).astype(np.float32)
    n = vals.size
    cl = ChunkLists([n], n + 5, alias=True)
    cl.set("p32", 0, vals)
    cl.set("m", 0, np.zeros(n, np.float32))
    cl.set("v", 0, np.zeros(n, np.float32))
    g = np.zeros(n, np.uint16)
    g[7] = 0x7C00                        # overflow: the step is skipped and the aliased chunk re-cast
    cl.set("g16", 0, g)
    hp = dict(step=1, loss_scale=1.0)
    psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
    flag, _ = psx.psx_overflow_read(ctx)
    assert flag == 1 == cl.oracle_step(orc, orc.hyper(**hp))
    assert cl.compare("recast") == 0.0
    with np.errstate(over="ignore"):
        assert np.array_equal(bits16(cl.p16[0])[:n], vals.astype(np.float16).view(np.uint16))


def test_fp16_recast_of_every_fp32_bit_pattern(orc, ctx):
    """All 2^32 fp32 bit patterns through the kernels' fp32 -> fp16 conversion (the skipped-step re-cast of a
    reused fp16 chunk), in windows of 2^28, bit for bit against the oracle's conversion.  NaN inputs are
    compared by class: the result must be a NaN of the same sign (which payload bits survive is not
    part of the format's rounding rule)."""
    from concurrent.futures import ThreadPoolExecutor
    W28 = 1 << 28
    p32 = torch.empty(W28, dtype=torch.int32, device=DEV)
    m = torch.zeros(W28, dtype=torch.float32, device=DEV)
    h16 = torch.empty(W28, dtype=torch.int16, device=DEV)
    idx = torch.arange(W28, dtype=torch.int64, device=DEV)
    spec = [dict(g16=h16, p16=h16, p32=p32, m=m, v=m, used=W28)]      # m and v are never written on a skipped step
    chunks = psx.make_chunks(spec)
    parts = 16
    pool = ThreadPoolExecutor(parts)
    for win in range(16):
        base = win * W28
        p32.copy_((idx + base).to(torch.int32))                       # wraps into the negative half: the bit pattern counts
        h16.zero_()
        h16[12345] = 0x7C00                                           # an inf gradient: the step is skipped, p16 = fp16(p32)
        psx.psx_chunk_adam_step(ctx, chunks, psx.make_hyper(step=1, loss_scale=1.0), psx.PSX_STEP_CHECK_FIRST)
        flag, _ = psx.psx_overflow_read(ctx)
        assert flag == 1
        got = h16.cpu().numpy().view(np.uint16)
        bits = np.arange(base, base + W28, dtype=np.uint64).astype(np.uint32)
        step = W28 // parts
        want = np.concatenate(list(pool.map(lambda j: orc.f32_to_f16(bits[j * step:(j + 1) * step].view(np.float32)), range(parts))))
        isnan = (bits & 0x7FFFFFFF) > 0x7F800000
        assert np.array_equal(got[~isnan], want[~isnan]), f"window {win}: {np.count_nonzero(got[~isnan] != want[~isnan])} differ"
        if isnan.any():
            g = got[isnan]
            assert np.all((g & 0x7C00) == 0x7C00) and np.all((g & 0x03FF) != 0), f"window {win}: a NaN became a number"
            assert np.array_equal(g & 0x8000, ((bits[isnan] >> 16) & 0x8000).astype(np.uint16)), f"window {win}: NaN sign"
    assert not m.any()
    pool.shutdown()


# ---------------------------------------------------------------------------------- skip semantics

@pytest.mark.parametrize("alias", [False, True])
def test_overflow_skips_the_whole_step(orc, ctx, alias):
    used = [20000, 12289, 1, 4097]
    Cn = 20000
    for (k, pos, special) in [(0, 0, 0x7C00), (1, 12288, 0xFC00), (2, 0, 0x7E00), (3, 4096, 0x7D01)]:
        cl = ChunkLists(used, Cn, alias=alias)
        fill_state(cl, 7000, 1024.0, zero_mv=False)
        cl.set("g16", k, np.array([special], np.uint16), at=pos)
        before = [bits32(x).copy() for x in cl.p32 + cl.m + cl.v]
        hp = dict(lr=1e-3, weight_decay=0.01, step=5, loss_scale=1024.0)
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
        flag, per = psx.psx_overflow_read(ctx, len(used))
        assert flag == 1 == cl.oracle_step(orc, orc.hyper(**hp))
        assert per[k] == 1 and sum(per) == 1
        assert cl.compare("skipped") == 0.0
        for a, b in zip(cl.p32 + cl.m + cl.v, before):       # fp32 states keep their bits
            assert bits32(a).tobytes() == b.tobytes()
    # a special value in the padding does not skip
    cl = ChunkLists(used, Cn, alias=False)
    fill_state(cl, 7100, 1024.0)
    cl.set("g16", 1, np.array([0x7C00], np.uint16), at=12289)
    hp = dict(step=1, loss_scale=1024.0)
    psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
    flag, _ = psx.psx_overflow_read(ctx)
    assert flag == 0 == cl.oracle_step(orc, orc.hyper(**hp))
    assert cl.compare("padding special") == 0.0


# ---------------------------------------------------------------------------------- host-resident chunks

@pytest.mark.parametrize("slots,mode", [(2, 0), (3, 0), (3, 1)])
@pytest.mark.parametrize("alias", [False, True])
def test_host_resident_chunks_stream_through_staging(orc, alias, slots, mode):
    """mode 0: staged H2D / kernel / D2H; mode 1: the kernel works on the pinned buffers over the link."""
    ctx = psx.psx_ctx_create(max_chunks=64, max_tensors=16, staging_tile_elems=4096, staging_slots=slots)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_MODE, mode)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_GRID, 7)
    try:
        used = [20000, 4096, 12289, 1, 4097, 0, 16384, 9000]
        loc = [(G, G), (H, H), (H, H), (H, H), (H, G), (H, H), (G, H), (H, H)]
        Cn = 20000
        cl = ChunkLists(used, Cn, alias=alias)
        fill_state(cl, 8000, 65536.0, zero_mv=False)
        host = []
        for k in range(cl.n):
            hs = [torch.from_numpy(sent32(Cn)).pin_memory() for _ in range(3)]
            if loc[k][0] == H:          # the state starts on the host; the device copy is garbage
                for hbuf, name in zip(hs, ("p32", "m", "v")):
                    hbuf.copy_(torch.from_numpy(cl.np[name][k]))
                    if loc[k][1] == H:
                        getattr(cl, name)[k].view(torch.int32).fill_(0x0BADBEEF)
            host.append(hs)
        for t in (1, 2, 3):
            hp = dict(lr=1e-3, weight_decay=0.01, step=t, loss_scale=65536.0)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=loc, host=host)), psx.make_hyper(**hp),
                                    psx.PSX_STEP_CHECK_FIRST)
            torch.cuda.synchronize()
            assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
            where = [host[k] if loc[k][1] == H else None for k in range(cl.n)]
            assert cl.compare(f"t={t}", where=where) == 0.0
            tm = psx.psx_ctx_get_timing(ctx)
            assert tm.spill_elems == sum(u for u, l in zip(used, loc) if l != (G, G))
            assert tm.h2d_bytes == 12 * sum(u for u, l in zip(used, loc) if l[0] == H)
            assert tm.d2h_bytes == 12 * sum(u for u, l in zip(used, loc) if l[1] == H)
            # the next step finds the state where this one left it
            loc = [(b, b) for (_, b) in loc]
            for k in range(cl.n):
                cl.set("g16", k, W.grads_f16_np(used[k], 8500 + 10 * k + t, 65536.0))
    finally:
        psx.psx_ctx_destroy(ctx)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("alias", [False, True])
def test_skipped_step_still_moves_chunks_that_change_residence(orc, alias, mode):
    """An overflow skips the update, but a chunk admitted to or evicted from HBM in that step must still
    find its fp32 states, bit for bit, in the new home; aliased fp16 chunks get their parameters back.
    Direct mode needs no staging at all, so its context is created without any."""
    ctx = psx.psx_ctx_create(max_chunks=8, max_tensors=4, staging_tile_elems=4096 if mode == 0 else 0, staging_slots=2)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_MODE, mode)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_GRID, 5)
    try:
        used = [5000, 4097, 1, 9000, 12288]
        loc = [(G, G), (H, G), (G, H), (H, H), (G, H)]
        Cn = 12288
        cl = ChunkLists(used, Cn, alias=alias)
        fill_state(cl, 8800, 1024.0, zero_mv=False)
        host = []
        for k in range(cl.n):
            hs = [torch.from_numpy(sent32(Cn)).pin_memory() for _ in range(3)]
            if loc[k][0] == H:
                for hbuf, name in zip(hs, ("p32", "m", "v")):
                    hbuf.copy_(torch.from_numpy(cl.np[name][k]))
                    getattr(cl, name)[k][:used[k]].view(torch.int32).fill_(0x0BADBEEF)    # device copy is garbage
            host.append(hs)
        cl.set("g16", 3, np.array([0xFC00], np.uint16), at=8999)
        hp = dict(lr=1e-3, weight_decay=0.01, step=3, loss_scale=1024.0)
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=loc, host=host)), psx.make_hyper(**hp),
                                psx.PSX_STEP_CHECK_FIRST)
        flag, per = psx.psx_overflow_read(ctx, len(used))
        torch.cuda.synchronize()
        assert flag == 1 == cl.oracle_step(orc, orc.hyper(**hp)) and list(per) == [0, 0, 0, 1, 0]
        where = [host[k] if loc[k][1] == H else None for k in range(cl.n)]
        assert cl.compare("skipped, moved", where=where) == 0.0
        # and the step after it, now finite, runs from the new homes
        cl.set("g16", 3, np.array([0x3C00], np.uint16), at=8999)
        if alias:                                    # the fp16 chunks hold parameters again: new gradients
            for k in range(cl.n):
                cl.set("g16", k, W.grads_f16_np(used[k], 8900 + k, 1024.0))
        loc = [(b, b) for (_, b) in loc]
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=loc, host=host)), psx.make_hyper(**hp),
                                psx.PSX_STEP_CHECK_FIRST)
        torch.cuda.synchronize()
        assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
        assert cl.compare("after the skipped step", where=where) == 0.0
    finally:
        psx.psx_ctx_destroy(ctx)


def test_bad_arguments_touch_nothing():
    ctx = psx.psx_ctx_create(max_chunks=4, max_tensors=4)
    try:
        cl = ChunkLists([64], 64)
        fill_state(cl, 1, 1.0)
        hs = [torch.zeros(64).pin_memory() for _ in range(3)]
        # staged host-resident chunks, and chunks changing residence, need a context with staging
        psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_MODE, 0)
        with pytest.raises(psx.PsxError) as e:
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=[(H, H)], host=[hs])), psx.make_hyper())
        assert e.value.code == psx.PSX_ENOSTAGING
        with pytest.raises(psx.PsxError) as e:
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=[(H, G)], host=[hs])), psx.make_hyper())
        assert e.value.code == psx.PSX_ENOSTAGING
        psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_MODE, 1)
        # direct access to host states that are not page-locked would fault the GPU: refused up front
        pageable = [torch.zeros(64) for _ in range(3)]
        with pytest.raises(psx.PsxError) as e:
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs(loc=[(H, H)], host=[pageable])), psx.make_hyper())
        assert e.value.code == psx.PSX_EINVAL and "not pinned" in str(e.value)
        with pytest.raises(psx.PsxError) as e:      # misaligned chunk base
            bad = cl.specs()
            bad[0]["p32"] = cl.p32[0].data_ptr() + 4
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(bad), psx.make_hyper())
        assert e.value.code == psx.PSX_EALIGN
        with pytest.raises(psx.PsxError) as e:      # more chunks than the context holds
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs() * 5), psx.make_hyper())
        assert e.value.code == psx.PSX_ECAP
        with pytest.raises(psx.PsxError) as e:
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(cl.specs()), psx.make_hyper(step=0))
        assert e.value.code == psx.PSX_EINVAL
        slots, used = psx.psx_chunk_layout([64], 64)
        with pytest.raises(psx.PsxError) as e:      # slot running past the chunk list
            slots[0].numel = 65
            psx.psx_pack(ctx, psx.PSX_F32, [cl.m[0]], slots, [cl.p32[0]], 64)
        assert e.value.code == psx.PSX_EINVAL
        with pytest.raises(psx.PsxError) as e:      # fused check is for fp16 only
            slots[0].numel = 64
            psx.psx_pack(ctx, psx.PSX_F32, [cl.m[0]], slots, [cl.p32[0]], 64, flags=psx.PSX_PACK_CHECK_OVERFLOW)
        assert e.value.code == psx.PSX_EINVAL
        torch.cuda.synchronize()
        assert cl.compare("after refused calls") == 0.0       # nothing was touched
    finally:
        psx.psx_ctx_destroy(ctx)


# ---------------------------------------------------------------------------------- host-resident chunks on the host cores

@pytest.mark.parametrize("wd,adamw,isa", [(0.0, 0, 0), (0.01, 0, 0), (0.01, 1, 0), (0.01, 0, 1), (0.01, 1, 1)])
@pytest.mark.parametrize("alias", [False, True])
def test_host_chunks_updated_by_the_host_cores(orc, alias, wd, adamw, isa):
    """PSX_EXEC_CPU: the paper's placement for host-resident optimizer states.  Same bits as the GPU kernel
    and the oracle, mixed in one call with HBM-resident and GPU-updated host chunks; a skipped step too."""
    ctx = psx.psx_ctx_create(max_chunks=64, max_tensors=16, staging_tile_elems=4096, staging_slots=3)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_THREADS, 3)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_TILE_ELEMS, 4096)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_ISA, isa)      # 0: AVX-512 where the host has it; 1: AVX2
    try:
        used = [20000, 4096, 12289, 1, 4097, 0, 16384, 9007, 15]
        loc = [(G, G), (H, H), (H, H), (H, H), (H, H), (H, H), (G, G), (H, H), (H, H)]
        ex = [0, 1, 1, 1, 0, 1, 0, 1, 1]
        Cn = 20000
        cl = ChunkLists(used, Cn, alias=alias)
        fill_state(cl, 9000, 65536.0, zero_mv=False)
        cl.set("g16", 7, np.array([0, 0x8000, 1, 0x8001, 0x03FF, 0x7BFF, 0xFBFF, 0x0400], np.uint16))
        host = []
        for k in range(cl.n):
            hs = None
            if loc[k][0] == H:
                hs = [psx.PinnedF32(Cn, fill=0.0) for _ in range(3)]
                for hbuf, name in zip(hs, ("p32", "m", "v")):
                    hbuf.np[...] = cl.np[name][k]
                    getattr(cl, name)[k].view(torch.int32).fill_(0x0BADBEEF)
            host.append(hs)
        specs = cl.specs(loc=loc, host=host)
        for s, e in zip(specs, ex):
            s["exec"] = e

        class HostView:                       # lets ChunkLists.compare read the pinned buffers
            def __init__(self, b): self.b = b
            def cpu(self): return self
            def numpy(self): return self.b.np
        where = [None if h is None else [HostView(b) for b in h] for h in host]
        for t in (1, 2, 3):
            if t == 3:                        # an overflow in a GPU-resident chunk skips the host-core update too
                cl.set("g16", 0, np.array([0x7C00], np.uint16), at=19999)
            hp = dict(lr=1e-3, weight_decay=wd, adamw_mode=adamw, step=t, loss_scale=65536.0)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(specs), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
            flag, _ = psx.psx_overflow_read(ctx)
            torch.cuda.synchronize()
            assert flag == cl.oracle_step(orc, orc.hyper(**hp)) == int(t == 3)
            assert cl.compare(f"t={t}", where=where) == 0.0
            tm = psx.psx_ctx_get_timing(ctx)
            assert tm.cpu_elems == sum(u for u, e in zip(used, ex) if e) and tm.cpu_threads == 3
            assert tm.spill_elems == used[4]
            if t < 3:
                for k in range(cl.n):
                    cl.set("g16", k, W.grads_f16_np(used[k], 9500 + 10 * k + t, 65536.0))
        # asking for the host cores on a chunk that lives in HBM is refused
        bad = cl.specs()
        bad[0]["exec"] = psx.PSX_EXEC_CPU
        with pytest.raises(psx.PsxError) as e:
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(bad), psx.make_hyper())
        assert e.value.code == psx.PSX_EINVAL
    finally:
        psx.psx_ctx_destroy(ctx)
        for hs in host:
            for b in hs or []:
                b.free()


def test_step_on_a_side_stream_orders_itself_with_that_stream(orc):
    """Everything a call starts on the context's own streams is joined back into the caller's stream:
    synchronising that stream alone (not the device) must show the finished step, host chunks included."""
    ctx = psx.psx_ctx_create(max_chunks=16, max_tensors=4, staging_tile_elems=4096, staging_slots=2)
    side = torch.cuda.Stream()
    host = []
    try:
        used = [20000, 12289, 4097, 9000, 16000]
        loc = [(G, G), (H, H), (H, H), (G, H), (H, G)]
        ex = [0, 0, 1, 0, 0]
        Cn = 20000
        cl = ChunkLists(used, Cn)
        fill_state(cl, 9900, 1024.0, zero_mv=False)
        for k in range(cl.n):
            hs = [psx.PinnedF32(Cn, fill=0.0) for _ in range(3)]
            if loc[k][0] == H:
                for hbuf, name in zip(hs, ("p32", "m", "v")):
                    hbuf.np[...] = cl.np[name][k]
                    getattr(cl, name)[k].view(torch.int32).fill_(0x0BADBEEF)
            host.append(hs)
        torch.cuda.synchronize()
        specs = cl.specs(loc=loc, host=host)
        for s, e in zip(specs, ex):
            s["exec"] = e
        hp = dict(lr=1e-3, weight_decay=0.01, step=4, loss_scale=1024.0)
        with torch.cuda.stream(side):
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(specs), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
            out = [cl.p16[k].clone() for k in range(cl.n)]            # queued on the same stream, after the step
        side.synchronize()
        assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
        for k in range(cl.n):
            u = used[k]
            assert np.array_equal(bits16(out[k])[:u], cl.np["p16"][k][:u])
            for j, name in enumerate(("p32", "m", "v")):
                got = host[k][j].np if loc[k][1] == H else f32(getattr(cl, name)[k])
                assert got[:u].tobytes() == cl.np[name][k][:u].tobytes(), (k, name)
    finally:
        torch.cuda.synchronize()
        psx.psx_ctx_destroy(ctx)
        for hs in host:
            for b in hs:
                b.free()


def test_two_contexts_on_two_streams_at_once(orc):
    """Two contexts, each with its own stream and chunk lists (one of them partly host-resident), stepping
    at the same time for several steps without a device-wide synchronisation in between: each sequence
    of steps must come out as if it had run alone."""
    ctxs = [psx.psx_ctx_create(max_chunks=8, max_tensors=4, staging_tile_elems=4096, staging_slots=2) for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    host = []
    try:
        Cn = 150000
        used = [[150000, 70001, 12345], [99999, 150000, 1, 4096]]
        locs = [[(G, G)] * 3, [(G, G), (H, H), (G, G), (H, H)]]
        cls, specs = [], []
        for j in range(2):
            cl = ChunkLists(used[j], Cn)
            fill_state(cl, 4400 + j, 512.0, zero_mv=False)
            hs_all = []
            for k in range(cl.n):
                hs = [psx.PinnedF32(Cn, fill=0.0) for _ in range(3)]
                if locs[j][k][0] == H:
                    for hbuf, name in zip(hs, ("p32", "m", "v")):
                        hbuf.np[...] = cl.np[name][k]
                        getattr(cl, name)[k].view(torch.int32).fill_(0x0BADBEEF)
                hs_all.append(hs)
            host.append(hs_all)
            cls.append(cl)
            specs.append(cl.specs(loc=locs[j], host=hs_all))
        torch.cuda.synchronize()
        hps = [dict(lr=1e-3, weight_decay=0.01, loss_scale=512.0), dict(lr=3e-4, beta1=0.8, beta2=0.99, weight_decay=0.1, adamw_mode=1, loss_scale=512.0)]
        steps = 4
        for t in range(1, steps + 1):
            for j in range(2):
                with torch.cuda.stream(streams[j]):
                    psx.psx_chunk_adam_step(ctxs[j], psx.make_chunks(specs[j]), psx.make_hyper(step=t, **hps[j]), psx.PSX_STEP_CHECK_FIRST)
        for st in streams:
            st.synchronize()
        for j in range(2):
            for t in range(1, steps + 1):
                assert cls[j].oracle_step(orc, orc.hyper(step=t, **hps[j])) == 0
            for k in range(cls[j].n):
                u = used[j][k]
                assert np.array_equal(bits16(cls[j].p16[k])[:u], cls[j].np["p16"][k][:u]), (j, k)
                for i, name in enumerate(("p32", "m", "v")):
                    got = host[j][k][i].np if locs[j][k][1] == H else f32(getattr(cls[j], name)[k])
                    assert got[:u].tobytes() == cls[j].np[name][k][:u].tobytes(), (j, k, name)
    finally:
        torch.cuda.synchronize()
        for c in ctxs:
            psx.psx_ctx_destroy(c)
        for hs_all in host:
            for hs in hs_all:
                for b in hs:
                    b.free()


@pytest.mark.parametrize("exec_cpu", [0, 1])
def test_fp32_denormals_are_kept(orc, exec_cpu):
    """A huge loss scale with tiny gradients drives g, m, v and the products on the way through the fp32
    denormal range; the GPU kernel and the host-core kernel must keep denormals exactly as the oracle does."""
    ctx = psx.psx_ctx_create(max_chunks=4, max_tensors=4)
    host = None
    try:
        n = 70000
        rng = np.random.default_rng(123)
        g = rng.integers(0, 0x0C00, size=n).astype(np.uint16)            # fp16 subnormals and the smallest normals
        g |= (rng.integers(0, 2, size=n).astype(np.uint16) << 15)
        cl = ChunkLists([n], n + 3)
        cl.set("g16", 0, g)
        cl.set("p32", 0, W.params_np(n, 77) * np.float32(1e-30))         # params near the denormal range too
        tiny = (rng.random(n, dtype=np.float32) * np.float32(1e-38)).astype(np.float32)
        cl.set("m", 0, tiny * np.float32(0.3) * np.where(rng.random(n) < 0.5, -1, 1).astype(np.float32))
        cl.set("v", 0, tiny)
        assert np.any((np.abs(cl.np["v"][0][:n]) < 1.1754944e-38) & (cl.np["v"][0][:n] != 0))
        loc, hostbufs = None, None
        if exec_cpu:
            host = [psx.PinnedF32(n) for _ in range(3)]
            for hbuf, name in zip(host, ("p32", "m", "v")):
                hbuf.np[...] = cl.np[name][0][:n]
            loc, hostbufs = [(H, H)], [host]
        specs = cl.specs(loc=loc, host=hostbufs)
        specs[0]["exec"] = exec_cpu

        class HostView:
            def __init__(self, b): self.b = b
            def cpu(self): return self
            def numpy(self): return np.concatenate([self.b.np, cl.np["p32"][0][n:]])     # padding as in the mirror
        where = [[HostView(b) for b in host]] if exec_cpu else None
        for t, scale in ((1, 2.0 ** 40), (2, 2.0 ** 36), (3, 2.0 ** 44)):
            hp = dict(lr=1e-3, eps=1e-30, weight_decay=0.0, step=t, loss_scale=scale)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(specs), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
            torch.cuda.synchronize()
            assert cl.oracle_step(orc, orc.hyper(**hp)) == 0
            assert cl.compare(f"t={t}", where=where) == 0.0
            v_now = cl.np["v"][0][:n]
            if t == 1:                                              # denormals really occur
                assert np.count_nonzero((v_now != 0) & (np.abs(v_now) < 1.1754944e-38)) > 100
    finally:
        psx.psx_ctx_destroy(ctx)
        for b in host or []:
            b.free()
