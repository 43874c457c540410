"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py times.
The oracle cannot run 10^9 elements in seconds, so it runs free on a sample of
whole chunks (first, last, the one holding the tail of the oversized embedding,
the emptiest, random others), fed with the same seeded tensors; sampled chunks
must match bit for bit.  Properties that hold at any size (skip leaves state
untouched, scaler halves) cover what the sample cannot."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import bench
from paper_2108_05818_amd import psx
from paper_2108_05818_amd import workloads as W

from gpu_util import DEV, bits16, f32, from_bits16

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _release_cached_device_memory():
    """These tests allocate tens to hundreds of GB; start each from an empty allocator cache."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    yield
    gc.collect()
    torch.cuda.empty_cache()


class Sample:
    """Oracle-side mirror of a subset of chunks of a bench.State, built only from the seeded tensors."""

    def __init__(self, orc, st, ks):
        self.orc, self.st, self.ks = orc, st, sorted(set(ks))
        w, C = st.w, st.C
        self.o_slots, self.o_used = orc.chunk_layout(w.numel, C)
        assert [int(u) for u in self.o_used] == st.used
        nch = st.nch
        mk = lambda dt: [np.zeros(C, dt) if k in self.ks else None for k in range(nch)]
        self.p32, self.m, self.v, self.p16, self.g16 = mk(np.float32), mk(np.float32), mk(np.float32), mk(np.uint16), mk(np.uint16)
        # tensors that overlap a sampled chunk
        self.idx = []
        for i, s in enumerate(w.numel):
            if s == 0:
                continue
            lo = self.o_slots[i].chunk * C + self.o_slots[i].offset
            if any(lo < (k + 1) * C and lo + s > k * C for k in self.ks):
                self.idx.append(i)
        self.sub_slots = (orc.Slot * len(self.idx))(*[self.o_slots[i] for i in self.idx])
        self.pool = ThreadPoolExecutor(min(8, len(self.ks)))

    def pack(self, tensors_dev, into, as_bits16=False):
        host = [bits16(tensors_dev[i]) if as_bits16 else f32(tensors_dev[i]) for i in self.idx]
        self.orc.pack(host, self.sub_slots, into, self.st.C)

    def adam(self, h):
        used = self.st.used
        list(self.pool.map(lambda k: self.orc.adam_chunk(self.g16[k], self.p16[k], self.p32[k], self.m[k], self.v[k],
                                                         used[k], h), self.ks))

    def flag(self):
        ks = self.ks
        return self.orc.overflow_check([self.g16[k] for k in ks], np.array([self.st.used[k] for k in ks], np.uint64))[0]

    def compare(self, tag):
        st = self.st
        for k in self.ks:
            for name, dev, mine in (("p32", st.p32[k], self.p32[k]), ("m", st.m[k], self.m[k]), ("v", st.v[k], self.v[k])):
                assert f32(dev).tobytes() == mine.tobytes(), f"{tag}: chunk {k} {name}"
            assert bits16(st.p16[k]).tobytes() == self.p16[k].tobytes(), f"{tag}: chunk {k} p16"
            assert bits16(st.g16[k]).tobytes() == self.g16[k].tobytes(), f"{tag}: chunk {k} g16"

    def compare_unpacked(self, tag):
        """fp16 tensors that lie wholly inside sampled chunks, against the oracle's unpack."""
        st, C = self.st, self.st.C
        inside = [i for i in self.idx
                  if all((p // C) in self.ks for p in (self.o_slots[i].chunk * C + self.o_slots[i].offset,
                                                      self.o_slots[i].chunk * C + self.o_slots[i].offset + st.w.numel[i] - 1))
                  and st.w.numel[i] <= C]
        outs = [np.zeros(st.w.numel[i], np.uint16) for i in inside]
        self.orc.unpack(outs, (self.orc.Slot * len(inside))(*[self.o_slots[i] for i in inside]), self.p16, C)
        for i, o in zip(inside, outs):
            assert bits16(st.out_t[i]).tobytes() == o.tobytes(), f"{tag}: tensor {i}"
        return len(inside)


def snapshot(st, ks):
    return {k: [x.clone() for x in (st.p32[k], st.m[k], st.v[k], st.p16[k])] for k in ks}


def assert_unchanged(st, snap, tag):
    for k, bufs in snap.items():
        for a, b in zip((st.p32[k], st.m[k], st.v[k], st.p16[k]), bufs):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"{tag}: chunk {k} changed"


def test_config2_gpt1b_full_size_sampled_chunks(orc):
    w = W.config2_gpt1b()
    st = bench.setup(w, DEV)
    try:
        assert st.nch == 44 and w.n_elems == 1112193024
        emptiest = int(np.argmin(st.used))
        ks = [0, 3, st.nch - 1, emptiest, 17]
        sm = Sample(orc, st, ks)
        sm.pack(st.p_t, sm.p32)
        sm.compare("after param pack")
        o_scaler = orc.scaler(w.loss_scale, w.growth_interval)
        for step in range(2):
            flag = bench.run_step(st)                 # pack grads, check, Adam, unpack, flag, scaler
            torch.cuda.synchronize()
            sm.pack(st.g_t, sm.g16, as_bits16=True)
            assert flag == sm.flag() == 0
            sm.adam(orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                              adamw_mode=w.adamw_mode, step=o_scaler.step, loss_scale=o_scaler.scale))
            orc.scaler_update(o_scaler, 0)
            sm.compare(f"step {step}")
            assert sm.compare_unpacked(f"step {step}") > 0
            assert (st.scaler.scale, st.scaler.step) == (o_scaler.scale, o_scaler.step)
        # an inf planted in one gradient element far from the sample: the whole step is skipped
        victim = next(i for i in range(len(w.numel) - 1, 0, -1) if i not in sm.idx and w.numel[i] > 1000)
        saved = st.g_t[victim][777].clone()
        st.g_t[victim][777] = float("inf")
        every = snapshot(st, range(st.nch))
        flag = bench.run_step(st)
        torch.cuda.synchronize()
        assert flag == 1
        assert_unchanged(st, every, "skipped step")
        orc.scaler_update(o_scaler, 1)
        assert (st.scaler.scale, st.scaler.step) == (o_scaler.scale, o_scaler.step) == (w.loss_scale / 2, 3)
        st.g_t[victim][777] = saved
        # and the fused pack+check form of the step reaches the same state as the oracle
        del every
        flag = bench.run_step(st, fused_check=True)
        torch.cuda.synchronize()
        assert flag == 0
        sm.adam(orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                          adamw_mode=w.adamw_mode, step=o_scaler.step, loss_scale=o_scaler.scale))
        sm.compare("fused-check step")
    finally:
        psx.psx_ctx_destroy(st.ctx)


def test_config3_ragged_full_size_sampled_chunks(orc):
    w = W.config3_ragged()
    st = bench.setup(w, DEV)
    try:
        rng = np.random.default_rng(31)
        ks = [0, st.nch - 1] + [int(x) for x in rng.choice(np.arange(1, st.nch - 1), size=2, replace=False)]
        sm = Sample(orc, st, ks)
        sm.pack(st.p_t, sm.p32)
        sm.compare("after param pack")
        o_scaler = orc.scaler(w.loss_scale, 2)
        st.scaler.growth_interval = 2
        inject_at = {2: int(rng.integers(0, len(w.numel)))}
        for step in range(5):
            saved = None
            if step in inject_at:
                i = inject_at[step]
                pos = int(rng.integers(0, w.numel[i]))
                saved = (i, pos, st.g_t[i][pos].clone())
                st.g_t[i][pos] = float("nan")
                every = snapshot(st, sm.ks)
            # gradients are generated at the current scale only at set-up; what matters here is the unscale value
            flag = bench.run_step(st)
            torch.cuda.synchronize()
            if saved is not None:
                assert flag == 1
                assert_unchanged(st, every, "skipped step")
                st.g_t[saved[0]][saved[1]] = saved[2]
                orc.scaler_update(o_scaler, 1)
            else:
                sm.pack(st.g_t, sm.g16, as_bits16=True)
                assert flag == sm.flag() == 0
                sm.adam(orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                                  adamw_mode=w.adamw_mode, step=o_scaler.step, loss_scale=o_scaler.scale))
                orc.scaler_update(o_scaler, 0)
                sm.compare(f"step {step}")
                assert sm.compare_unpacked(f"step {step}") > 0
            assert (st.scaler.scale, st.scaler.step, st.scaler.good_steps) == \
                   (o_scaler.scale, o_scaler.step, o_scaler.good_steps)
        assert o_scaler.scale == w.loss_scale * 2          # doubled after 2 good steps, halved by the nan, doubled again
    finally:
        psx.psx_ctx_destroy(st.ctx)


def test_config3_scaled_down_200_steps_with_random_injection(orc):
    """Ragged sizes (log-uniform), 200 steps, every step compared in full with the free-running oracle;
    each step plants an inf/nan with probability 1% (seeded), plus three forced ones."""
    from gpu_util import ChunkLists
    w = W.config3_ragged(n=300, hi=16384, chunk_elems=65536)
    slots, used = psx.psx_chunk_layout(w.numel, w.chunk_elems)
    o_slots, _ = orc.chunk_layout(w.numel, w.chunk_elems)
    ctx = psx.psx_ctx_create(max_chunks=len(used), max_tensors=len(w.numel))
    try:
        cl = ChunkLists(used, w.chunk_elems)
        p_np = [W.params_np(s, 3000 + i) for i, s in enumerate(w.numel)]
        psx.psx_pack(ctx, psx.PSX_F32, [torch.from_numpy(a).to(DEV) for a in p_np], slots, cl.p32, w.chunk_elems)
        orc.pack(p_np, o_slots, cl.np["p32"], w.chunk_elems)
        for k in range(cl.n):
            cl.set("m", k, np.zeros(used[k], np.float32))
            cl.set("v", k, np.zeros(used[k], np.float32))
        scaler, o_scaler = psx.make_scaler(w.loss_scale, w.growth_interval), orc.scaler(w.loss_scale, w.growth_interval)
        rng = np.random.default_rng(3001)
        chunks = psx.make_chunks(cl.specs())
        skipped = doubled = 0
        for step in range(200):
            g_np = [W.grads_f16_np(s, 7000 + 1000 * step + i, scaler.scale) for i, s in enumerate(w.numel)]
            if rng.random() < w.inject_prob or step in (5, 60, 61):
                i = int(rng.integers(0, len(w.numel)))
                g_np[i][int(rng.integers(0, w.numel[i]))] = rng.choice(W.specials_f16())
            psx.psx_overflow_reset(ctx)
            psx.psx_pack(ctx, psx.PSX_F16, [from_bits16(a) for a in g_np], slots, cl.g16, w.chunk_elems,
                         flags=psx.PSX_PACK_CHECK_OVERFLOW)
            orc.pack(g_np, o_slots, cl.np["g16"], w.chunk_elems)
            hp = dict(lr=w.lr, weight_decay=w.weight_decay, step=scaler.step, loss_scale=scaler.scale)
            psx.psx_chunk_adam_step(ctx, chunks, psx.make_hyper(**hp), psx.PSX_STEP_USE_FLAG)
            flag, per = psx.psx_overflow_read(ctx, cl.n)
            o_flag = cl.oracle_step(orc, orc.hyper(**hp))
            assert flag == o_flag
            assert per == list(orc.overflow_check(cl.np["g16"], np.array(used, np.uint64))[1])
            skipped += flag
            if step % 10 == 0 or flag or step == 199:
                assert cl.compare(f"step {step}") == 0.0
            before = scaler.scale
            psx.psx_loss_scale_update(scaler, flag)
            orc.scaler_update(o_scaler, o_flag)
            doubled += scaler.scale > before
            assert (scaler.scale, scaler.step, scaler.good_steps) == (o_scaler.scale, o_scaler.step, o_scaler.good_steps)
        assert skipped >= 3 and scaler.step == 201 - skipped
        assert doubled >= 1                                          # halvings and doublings both happened
    finally:
        psx.psx_ctx_destroy(ctx)


# ---------------------------------------------------------------------------------- host-resident chunks at real shapes

H, G = psx.PSX_LOC_HOST, psx.PSX_LOC_HBM


def compare_sample_states(sm, st, where, tag):
    """Sampled chunks against the oracle mirror, reading each chunk's states where they live now:
    `where[k]` is None (device) or the three pinned buffers (used prefix only)."""
    for k in sm.ks:
        u = st.used[k]
        for j, (name, mine) in enumerate((("p32", sm.p32[k]), ("m", sm.m[k]), ("v", sm.v[k]))):
            if where[k] is None:
                got = f32((st.p32[k], st.m[k], st.v[k])[j])
                assert got[u:].tobytes() == mine[u:].tobytes(), f"{tag}: chunk {k} {name} padding"
            else:
                got = where[k][j].np
            assert got[:u].tobytes() == mine[:u].tobytes(), f"{tag}: chunk {k} {name}"
        assert bits16(st.p16[k]).tobytes() == sm.p16[k].tobytes(), f"{tag}: chunk {k} p16"


@pytest.mark.parametrize("mode", [1, 0])
def test_config4_shape_host_resident_chunks(orc, mode):
    """GPT-12.6B tensor shapes (hidden 5120, 64 Mi chunks) at 4 layers; the last 40 % of the chunks keep
    their fp32 states in pinned host memory.  mode 1: kernel works over the link; mode 0: staged copies."""
    w = W.config4_gpt12b(layers=4)
    st = bench.setup(w, DEV, host_fraction=0.4)
    try:
        psx.psx_ctx_set_tuning(st.ctx, psx.PSX_TUNE_HOST_MODE, mode)
        first_host = st.nch - st.n_host
        assert st.n_host == round(0.4 * st.nch) and st.host[first_host] is not None and st.host[first_host - 1] is None
        sm = Sample(orc, st, [0, first_host - 1, first_host, st.nch - 1])
        sm.pack(st.p_t, sm.p32)
        where = [None if st.host[k] is None else st.host[k] for k in range(st.nch)]
        compare_sample_states(sm, st, where, "after param pack")
        for step in range(2):
            flag = bench.run_step(st)
            torch.cuda.synchronize()
            sm.pack(st.g_t, sm.g16, as_bits16=True)
            assert flag == sm.flag() == 0
            sm.adam(orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                              adamw_mode=w.adamw_mode, step=step + 1, loss_scale=w.loss_scale))
            compare_sample_states(sm, st, where, f"mode {mode} step {step}")
        tm = psx.psx_ctx_get_timing(st.ctx)
        host_elems = sum(st.used[first_host:])
        assert tm.spill_elems == host_elems and tm.h2d_bytes == tm.d2h_bytes == 12 * host_elems
    finally:
        psx.psx_ctx_destroy(st.ctx)
        for hs in st.host:
            for b in hs or []:
                b.free()


def test_config5_shape_residency_changes_every_step(orc):
    """GPT-20B tensor shapes (hidden 6144, 64 Mi chunks) at 2 layers.  The share of chunks whose fp32 states
    may stay in HBM moves by +-30 % per step (seeded), so chunks at the boundary of the resident prefix are
    admitted (HOST -> HBM) or evicted (HBM -> HOST) while they are updated; most chunks stay on the host."""
    w = W.config5_gpt20b(layers=2)
    st = bench.setup(w, DEV, host_fraction=0.0)          # device homes for every chunk; host homes added here
    ctx = psx.psx_ctx_create(max_chunks=st.nch, max_tensors=len(w.numel), staging_tile_elems=4 << 20, staging_slots=3)
    host = [[psx.PinnedF32(st.used[k]) for _ in range(3)] for k in range(st.nch)]
    try:
        nch = st.nch
        prefix = lambda t: max(1, min(nch - 1, round(nch * W.budget_fraction(t, 0.3, w.budget_jitter, w.seed))))
        r = prefix(0)
        sizes = [prefix(t) for t in range(1, 7)]
        assert len(set(sizes)) > 2 and max(sizes) < 0.5 * nch          # the boundary really moves; most chunks on host
        # initial residence: chunks >= r live on the host (their device homes are filled with garbage)
        for k in range(r, nch):
            for j, d in enumerate((st.p32[k], st.m[k], st.v[k])):
                host[k][j].np[...] = d[:st.used[k]].cpu().numpy()
                d.view(torch.int32).fill_(0x0BADBEEF)
        loc = [G if k < r else H for k in range(nch)]
        sm = Sample(orc, st, sorted({0, min(sizes) - 1, min(sizes), max(sizes) - 1, max(sizes), nch - 1}))
        sm.pack(st.p_t, sm.p32)
        slots, used = psx.psx_chunk_layout(w.numel, st.C)
        moved = 0
        for step in range(1, 7):
            r_new = prefix(step)
            new_loc = [G if k < r_new else H for k in range(nch)]
            moved += sum(a != b for a, b in zip(loc, new_loc))
            specs = [dict(g16=st.g16[k], p16=st.p16[k], p32=st.p32[k], m=st.m[k], v=st.v[k], used=st.used[k],
                          p32_host=host[k][0], m_host=host[k][1], v_host=host[k][2],
                          loc_in=loc[k], loc_out=new_loc[k]) for k in range(nch)]
            psx.psx_pack(ctx, psx.PSX_F16, st.g_t, slots, st.g16, st.C)
            hp = dict(lr=w.lr, weight_decay=w.weight_decay, step=step, loss_scale=w.loss_scale)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(specs), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
            flag, _ = psx.psx_overflow_read(ctx)
            torch.cuda.synchronize()
            # link bytes are exactly what the residency of this step implies, nothing is moved twice
            tm = psx.psx_ctx_get_timing(ctx)
            assert tm.h2d_bytes == 12 * sum(st.used[k] for k in range(nch) if loc[k] == H)
            assert tm.d2h_bytes == 12 * sum(st.used[k] for k in range(nch) if new_loc[k] == H)
            # evicted chunks: poison the device home so that a stale read would show
            for k in range(nch):
                if loc[k] == G and new_loc[k] == H:
                    for d in (st.p32[k], st.m[k], st.v[k]):
                        d.view(torch.int32).fill_(0x0BADBEEF)
            loc = new_loc
            if step == 1:
                sm.pack(st.g_t, sm.g16, as_bits16=True)
            assert flag == sm.flag() == 0
            sm.adam(orc.hyper(**hp))
            where = [None if loc[k] == G else host[k] for k in range(nch)]
            # device homes of sampled resident chunks were zero-initialised by the set-up, like the mirror
            for k in sm.ks:
                u = st.used[k]
                bufs = (st.p32[k], st.m[k], st.v[k]) if where[k] is None else None
                for j, mine in enumerate((sm.p32[k], sm.m[k], sm.v[k])):
                    got = f32(bufs[j])[:u] if bufs else where[k][j].np
                    assert got.tobytes() == mine[:u].tobytes(), f"step {step}: chunk {k} state {j}"
                assert bits16(st.p16[k]).tobytes() == sm.p16[k].tobytes(), f"step {step}: chunk {k} p16"
        assert moved >= 3
    finally:
        psx.psx_ctx_destroy(ctx)
        psx.psx_ctx_destroy(st.ctx)
        for hs in host:
            for b in hs:
                b.free()


# ---------------------------------------------------------------------------------- sizes past 2^31, and empty calls

def test_elements_beyond_two_to_the_31(orc):
    """One chunk with more than 2^31 elements in use, and one tensor of that size running over three chunks:
    every index in the kernels is 64-bit.  The oracle is run on windows at the start, across 2^31 and at the end."""
    n = (1 << 31) + 1000
    ctx = psx.psx_ctx_create(max_chunks=4, max_tensors=2)
    try:
        gen = torch.Generator(device=DEV)
        gen.manual_seed(77)
        g = torch.empty(n, dtype=torch.float16, device=DEV)
        p = torch.empty(n, dtype=torch.float32, device=DEV)
        step = 1 << 28
        for lo in range(0, n, step):                                  # fill piecewise to keep temporaries small
            hi = min(n, lo + step)
            g[lo:hi] = (torch.randn(hi - lo, generator=gen, device=DEV) * 65.0).half()
            p[lo:hi] = torch.randn(hi - lo, generator=gen, device=DEV) * 0.02
        m = torch.zeros(n, dtype=torch.float32, device=DEV)
        v = torch.zeros(n, dtype=torch.float32, device=DEV)
        p16 = torch.zeros(n, dtype=torch.float16, device=DEV)
        windows = [(0, 5000), ((1 << 31) - 3000, n), ((1 << 30) + 17, (1 << 30) + 4113), ((3 << 29) - 1, (3 << 29) + 2049)]
        before = [(bits16(g[a:b]), f32(p[a:b])) for a, b in windows]
        # overflow flag: clean, then an inf beyond 2^31
        flag, per = psx.psx_overflow_check(ctx, [g], [n])
        assert (flag, per) == (0, [0])
        keep = g[(1 << 31) + 500].clone()
        g[(1 << 31) + 500] = float("inf")
        assert psx.psx_overflow_check(ctx, [g], [n]) == (1, [1])
        assert psx.psx_overflow_check(ctx, [g], [(1 << 31) + 500]) == (0, [0])     # just outside the used prefix
        g[(1 << 31) + 500] = keep
        hp = dict(lr=1e-3, weight_decay=0.01, step=1, loss_scale=65536.0)
        spec = [dict(g16=g, p16=p16, p32=p, m=m, v=v, used=n)]
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(spec), psx.make_hyper(**hp), psx.PSX_STEP_CHECK_FIRST)
        torch.cuda.synchronize()
        for (a, b), (g_np, p_np) in zip(windows, before):
            k = b - a
            om, ov, o16 = np.zeros(k, np.float32), np.zeros(k, np.float32), np.zeros(k, np.uint16)
            op = p_np.copy()
            orc.adam_chunk(g_np.copy(), o16, op, om, ov, k, orc.hyper(**hp))
            assert f32(p[a:b]).tobytes() == op.tobytes() and f32(m[a:b]).tobytes() == om.tobytes()
            assert f32(v[a:b]).tobytes() == ov.tobytes() and bits16(p16[a:b]).tobytes() == o16.tobytes()
        # pack / unpack of a tensor with more than 2^31 elements over three chunks of 2^30
        C = 1 << 30
        slots, used = psx.psx_chunk_layout([5, n], C)
        assert used == [5, C, C, 1000] and (slots[1].chunk, slots[1].offset) == (1, 0)
        del m, v, p
        chunks = [torch.zeros(C, dtype=torch.float16, device=DEV) for _ in range(4)]
        five = torch.arange(5, dtype=torch.float16, device=DEV)
        psx.psx_pack(ctx, psx.PSX_F16, [five, g], slots, chunks, C)
        for (a, b) in windows:
            lin = C + a                                              # the tensor starts at chunk 1, offset 0
            got = torch.cat([chunks[(lin + i) // C][(lin + i) % C:(lin + i) % C + 1] for i in (0, b - a - 1)])
            assert torch.equal(got.view(torch.int16), torch.stack([g[a], g[b - 1]]).view(torch.int16))
        assert torch.equal(chunks[1].view(torch.int16), g[:C].view(torch.int16))
        assert torch.equal(chunks[3][:1000].view(torch.int16), g[2 * C:].view(torch.int16)) and not chunks[3][1000:].any()
        p16.zero_()
        psx.psx_unpack(ctx, psx.PSX_F16, [torch.zeros(5, dtype=torch.float16, device=DEV), p16], slots, chunks, C)
        torch.cuda.synchronize()
        assert torch.equal(p16.view(torch.int16), g.view(torch.int16))
    finally:
        psx.psx_ctx_destroy(ctx)


def test_empty_calls_do_nothing():
    ctx = psx.psx_ctx_create(max_chunks=4, max_tensors=4)
    try:
        assert psx.psx_overflow_check(ctx, [], []) == (0, [])
        psx.psx_chunk_adam_step(ctx, psx.make_chunks([]), psx.make_hyper(), psx.PSX_STEP_CHECK_FIRST, n_chunks=0)
        slots, used = psx.psx_chunk_layout([], 64)
        assert used == [0]
        c = torch.full((64,), 7.0, dtype=torch.float16, device=DEV)
        psx.psx_pack(ctx, psx.PSX_F16, [], slots, [c], 64, n=0)
        psx.psx_unpack(ctx, psx.PSX_F16, [], slots, [c], 64, n=0)
        # a list of empty tensors and a chunk with nothing in use
        slots, used = psx.psx_chunk_layout([0, 0], 64)
        e = torch.zeros(0, dtype=torch.float16, device=DEV)
        psx.psx_pack(ctx, psx.PSX_F16, [e, e], slots, [c], 64)
        z = torch.zeros(64, dtype=torch.float32, device=DEV)
        spec = [dict(g16=c, p16=c, p32=z, m=z, v=z, used=0)]
        psx.psx_chunk_adam_step(ctx, psx.make_chunks(spec), psx.make_hyper(), psx.PSX_STEP_CHECK_FIRST)
        assert psx.psx_overflow_read(ctx, 1) == (0, [0])
        torch.cuda.synchronize()
        assert torch.all(c == 7.0) and not z.any()
        r = psx.psx_measure_link(ctx, 16, 1)
        assert r.h2d_alone > 1.0 and r.d2h_alone > 1.0 and r.each_way_both > 0.5
    finally:
        psx.psx_ctx_destroy(ctx)


def test_config4_gpt12b_full_size_sampled_chunks(orc):
    """GPT-12.6B at full size (12.85 G elements, 244 chunks of 64 Mi), the last 98 chunks host-resident and
    updated over the link, exactly as `bench.py --workload gpt12b` runs it; oracle on four whole chunks."""
    import psutil
    if psutil.virtual_memory().available < 120 * (1 << 30) or torch.cuda.mem_get_info()[0] < 250 * (1 << 30):
        pytest.skip("needs 120 GiB of host memory and 250 GiB of HBM")
    w = W.config4_gpt12b()
    C = w.chunk_elems
    o_slots, o_used = orc.chunk_layout(w.numel, C)
    nch = len(o_used)
    first_host = nch - round(0.4 * nch)
    ks = [3, first_host - 1, first_host, nch - 1]
    needed = {i for i, s in enumerate(w.numel) if s and any(
        o_slots[i].chunk * C + o_slots[i].offset < (k + 1) * C and o_slots[i].chunk * C + o_slots[i].offset + s > k * C
        for k in ks)}
    st = bench.setup(w, DEV, host_fraction=0.4, keep_params=needed)
    try:
        assert st.nch == 244 and st.n_host == 98 and w.n_elems == 12848143360
        sm = Sample(orc, st, ks)
        assert set(sm.idx) == needed
        sm.pack(st.p_t, sm.p32)
        where = [None if st.host[k] is None else st.host[k] for k in range(st.nch)]
        compare_sample_states(sm, st, where, "after param pack")
        for step in range(2):
            flag = bench.run_step(st, fused_check=True)
            torch.cuda.synchronize()
            sm.pack(st.g_t, sm.g16, as_bits16=True)
            assert flag == sm.flag() == 0
            sm.adam(orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                              adamw_mode=w.adamw_mode, step=step + 1, loss_scale=w.loss_scale))
            compare_sample_states(sm, st, where, f"step {step}")
        tm = psx.psx_ctx_get_timing(st.ctx)
        assert tm.spill_elems == sum(st.used[first_host:]) == 5139102720
    finally:
        psx.psx_ctx_destroy(st.ctx)
        for hs in st.host:
            for b in hs or []:
                b.free()
