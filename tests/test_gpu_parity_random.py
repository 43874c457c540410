"""GPU parity on seeded random scenarios: random chunk fills, chunk reuse or not, every residency transition
and execution way mixed inside one call (HBM in place, host in place over the link or through staging, admitted,
evicted, host cores), random hyper-parameters, injected inf/nan on some steps.  Each step is compared in full with
the oracle, which runs free on its own mirror.  Everything stays inside its buffers by construction: `used` never
exceeds the chunk size the buffers were allocated with."""
import numpy as np
import pytest
import torch

from paper_2108_05818_amd import psx
from paper_2108_05818_amd import workloads as W

from gpu_util import ChunkLists, sent32

pytestmark = pytest.mark.gpu

H, G = psx.PSX_LOC_HOST, psx.PSX_LOC_HBM
POISON = 0x0BADBEEF


def _poison(buf, u):
    if u:
        buf[:u].view(torch.int32).fill_(POISON)


@pytest.mark.parametrize("seed", range(24))
def test_random_scenario(orc, seed):
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.integers(1, 9))
    Cn = int(rng.choice([1, 7, 1024, 4099, 12288, 20000]))
    picks = [0, 1, Cn, Cn - 1, Cn // 2, min(Cn, 1024), min(Cn, 1025), min(Cn, 255)]
    used = [int(max(0, rng.choice(picks))) if rng.random() < 0.5 else int(rng.integers(0, Cn + 1)) for _ in range(n)]
    alias = bool(rng.integers(0, 2))
    mode = int(rng.integers(0, 2))
    ctx = psx.psx_ctx_create(max_chunks=n, max_tensors=1, staging_tile_elems=int(rng.choice([64, 1024, 4096, 8200])),
                             staging_slots=int(rng.integers(2, 5)))
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_MODE, mode)
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_GRID, int(rng.integers(1, 41)))
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_HOST_UNROLL, int(rng.choice([1, 2, 4])))
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_THREADS, int(rng.integers(1, 5)))
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_TILE_ELEMS, int(rng.choice([16, 1024, 4096, 8208])))
    psx.psx_ctx_set_tuning(ctx, psx.PSX_TUNE_CPU_ISA, int(rng.integers(0, 2)))
    try:
        cl = ChunkLists(used, Cn, alias=alias)
        loss_scale = float(rng.choice([1.0, 1024.0, 65536.0]))
        for k in range(n):
            u = used[k]
            if u:
                cl.set("p32", k, W.params_np(u, 9100 + 50 * seed + k))
                cl.set("m", k, W.params_np(u, 9200 + 50 * seed + k) * np.float32(0.05))
                cl.set("v", k, np.abs(W.params_np(u, 9300 + 50 * seed + k)) * np.float32(1e-4))
        # every chunk has a pinned home too; the states start in either
        host = [[torch.from_numpy(sent32(Cn)).pin_memory() for _ in range(3)] for _ in range(n)]
        at = [int(rng.choice([G, H])) for _ in range(n)]
        for k in range(n):
            if at[k] == H:
                for hbuf, name in zip(host[k], ("p32", "m", "v")):
                    hbuf.copy_(torch.from_numpy(cl.np[name][k]))
                    _poison(getattr(cl, name)[k], used[k])
        t = 1
        for step in range(4):
            for k in range(n):
                if used[k]:
                    cl.set("g16", k, W.grads_f16_np(used[k], 9400 + 1000 * seed + 10 * step + k, loss_scale))
            inject = rng.random() < 0.3 and any(used)
            if inject:
                k = int(rng.choice([k for k in range(n) if used[k]]))
                cl.set("g16", k, np.array([rng.choice(W.specials_f16())], np.uint16), at=int(rng.integers(0, used[k])))
            flags = psx.PSX_STEP_CHECK_FIRST if inject or rng.random() < 0.8 else 0
            loc, execs = [], []
            for k in range(n):
                out = at[k] if rng.random() < 0.6 else int(rng.choice([G, H]))
                loc.append((at[k], out))
                execs.append(psx.PSX_EXEC_CPU if (at[k], out) == (H, H) and rng.random() < 0.4 else psx.PSX_EXEC_GPU)
            specs = cl.specs(loc=loc, host=host)
            for s, e in zip(specs, execs):
                s["exec"] = e
            hp = dict(lr=1e-3, weight_decay=float(rng.choice([0.0, 0.01])), adamw_mode=int(rng.integers(0, 2)),
                      step=t, loss_scale=loss_scale)
            psx.psx_chunk_adam_step(ctx, psx.make_chunks(specs), psx.make_hyper(**hp), flags)
            torch.cuda.synchronize()
            tag = f"seed {seed} step {step} (mode {mode}, alias {alias}, loc {loc}, exec {execs}, inject {inject})"
            o_flag = cl.oracle_step(orc, orc.hyper(**hp))
            assert o_flag == int(inject), tag
            if flags:
                assert psx.psx_overflow_read(ctx)[0] == o_flag, tag
            tm = psx.psx_ctx_get_timing(ctx)
            on_gpu = [e != psx.PSX_EXEC_CPU for e in execs]
            assert tm.h2d_bytes == 12 * sum(u for u, l, g in zip(used, loc, on_gpu) if l[0] == H and g), tag
            assert tm.d2h_bytes == 12 * sum(u for u, l, g in zip(used, loc, on_gpu) if l[1] == H and g), tag
            assert tm.cpu_elems == sum(u for u, g in zip(used, on_gpu) if not g), tag
            at = [l[1] for l in loc]
            assert cl.compare(tag, where=[host[k] if at[k] == H else None for k in range(n)]) == 0.0, tag
            # the home a chunk is not in is dead: make sure nobody reads it later
            for k in range(n):
                if loc[k][0] != loc[k][1]:
                    for name, hbuf in zip(("p32", "m", "v"), host[k]):
                        _poison(hbuf if at[k] == G else getattr(cl, name)[k], used[k])
            if not o_flag:
                t += 1
    finally:
        psx.psx_ctx_destroy(ctx)


@pytest.mark.parametrize("seed", range(16))
def test_random_pack_unpack(orc, seed):
    """Random tensor lists (empty, single-element and oversized tensors among them) at random chunk sizes,
    sources and destinations misaligned at random, every copy launch shape; the fp16 pack also takes the
    overflow test, with an inf/nan planted in some tensor on half of the seeds."""
    rng = np.random.default_rng(9900 + seed)
    f16 = bool(rng.integers(0, 2))
    dtype, npd, ipd, sent = (psx.PSX_F16, np.uint16, np.int16, 0x7E55) if f16 else (psx.PSX_F32, np.uint32, np.int32, 0x7FC12345)
    Cn = int(rng.choice([1, 2, 3, 64, 1000, 4096, 5003]))
    kinds = rng.integers(0, 6, size=int(rng.integers(1, 60)))
    numel = [int({0: 0, 1: 1, 2: rng.integers(1, Cn + 1), 3: Cn, 4: rng.integers(Cn + 1, 4 * Cn + 2),
                  5: rng.integers(1, 40)}[int(k)]) for k in kinds]
    ctx = psx.psx_ctx_create(max_chunks=512, max_tensors=64)
    for key, val in zip((psx.PSX_TUNE_COPY_THREADS, psx.PSX_TUNE_COPY_UNROLL, psx.PSX_TUNE_COPY_BLOCKS_PER_CU, psx.PSX_TUNE_NONTEMPORAL),
                        (int(rng.choice([64, 256])), int(rng.choice([0, 1, 4])), int(rng.choice([0, 0, 1, 3])), int(rng.integers(0, 2)))):
        psx.psx_ctx_set_tuning(ctx, key, val)
    try:
        slots, used = psx.psx_chunk_layout(numel, Cn)
        o_slots, o_used = orc.chunk_layout(numel, Cn)
        assert used == [int(u) for u in o_used]
        nch = len(used)
        if nch > 512:
            pytest.skip("more chunks than this context holds")
        gaps = [int(x) for x in rng.integers(0, 4, size=len(numel))]
        total = sum(numel) + sum(gaps) + 16
        big = rng.integers(0, 0x7BFF if f16 else 2 ** 32, size=total, dtype=np.uint64).astype(npd)   # finite halves
        planted = f16 and seed % 2 == 0 and sum(numel) > 0
        pos, spans = 1, []
        for s, gap in zip(numel, gaps):
            spans.append((pos, s))
            pos += s + gap
        if planted:
            i = int(rng.choice([i for i, s in enumerate(numel) if s]))
            big[spans[i][0] + int(rng.integers(0, numel[i]))] = rng.choice(W.specials_f16())
        big_t = torch.from_numpy(big.view(ipd)).to("cuda")
        t_np = [np.ascontiguousarray(big[p:p + s]) for p, s in spans]
        t_dev = [big_t[p:p + s] for p, s in spans]
        # chunks carved out of one arena at odd element offsets too, so destinations are misaligned as well
        cgap = [int(x) for x in rng.integers(0, 3, size=nch)]
        arena = torch.from_numpy(np.full(nch * Cn + sum(cgap) + 8, sent, npd).view(ipd)).to("cuda")
        cpos, chunks = 1, []
        for g in cgap:
            chunks.append(arena[cpos:cpos + Cn])
            cpos += Cn + g
        o_chunks = [np.full(Cn, sent, npd) for _ in range(nch)]
        flags = psx.PSX_PACK_CHECK_OVERFLOW if f16 else 0
        if flags:
            psx.psx_overflow_reset(ctx)
        psx.psx_pack(ctx, dtype, t_dev, slots, chunks, Cn, flags=flags)
        orc.pack(t_np, o_slots, o_chunks, Cn)
        torch.cuda.synchronize()
        for k in range(nch):
            assert chunks[k].cpu().numpy().view(npd).tobytes() == o_chunks[k].tobytes(), f"chunk {k}"
        # nothing between or around the chunks was written
        keep = np.ones(arena.numel(), bool)
        cpos = 1
        for g in cgap:
            keep[cpos:cpos + Cn] = False
            cpos += Cn + g
        assert (arena.cpu().numpy().view(npd)[keep] == sent).all()
        if flags:
            flag, per = psx.psx_overflow_read(ctx, nch)
            o_flag, o_per = orc.overflow_check(o_chunks, np.array(used, np.uint64))
            assert (flag, list(per)) == (o_flag, [int(x) for x in o_per]) and flag == int(planted)
        out_big = torch.zeros_like(big_t)
        outs = [out_big[p:p + s] for p, s in spans]
        psx.psx_unpack(ctx, dtype, outs, slots, chunks, Cn)
        torch.cuda.synchronize()
        mask = np.ones(total, bool)
        for (p, s), b in zip(spans, t_np):
            assert out_big[p:p + s].cpu().numpy().view(npd).tobytes() == b.tobytes()
            mask[p:p + s] = False
        assert not out_big.cpu().numpy()[mask].any()
    finally:
        psx.psx_ctx_destroy(ctx)
