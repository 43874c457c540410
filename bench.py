#!/usr/bin/env python3
"""Benchmark of the chunked mixed-precision Adam path on one MI355X.

A "step" is one pass of the whole hot path over the synthetic GPT-shaped
parameter set, every part of it in the HIP library behind include/psx.h:
  psx_chunk_layout (host)  ->  psx_pack of the fp16 gradients into their chunk
  slots, taking the inf/nan overflow test on the way (--separate-check runs it
  as a pass of its own over all gradient chunks instead)  ->  fused Adam over
  the chunk list (fp32 p/m/v updated, fp16 params written), skipped if the flag
  is set  ->  psx_unpack of the fp16 params  ->  flag read-back (4 bytes,
  synchronises) and loss-scale update.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps 20] [--warmup 3] [--workload gpt1b|tiny|gpt12b|ragged|gpt20b]
"""
import argparse
import ctypes
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

CPU_BASELINE_TENSORS = 64      # the oracle leg reads a prefix of the tensor list, never more than this
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
ADAM_BYTES_PER_ELEM = 28       # read g16 2 + p,m,v 12; write p,m,v 12 + p16 2


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt1b", choices=["gpt1b", "tiny", "gpt12b", "ragged", "gpt20b"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (shape-preserving scale-down)")
    ap.add_argument("--chunk-elems", type=int, default=0, help="override the chunk size (elements)")
    ap.add_argument("--host-fraction", type=float, default=-1.0, help="share of chunks whose fp32 states live in pinned host memory")
    ap.add_argument("--cpu-share", type=float, default=0.0, help="share of the host-resident chunks updated by the host cores instead of the GPU")
    ap.add_argument("--chunk-reuse", action="store_true",
                    help="the paper's chunk reuse: gradients are packed into the fp16 parameter chunks and overwritten "
                         "there by the new parameters (default: a gradient chunk list of its own)")
    ap.add_argument("--arena-skew", type=int, default=0, metavar="BYTES",
                    help="start chunk list j of the device arenas j*BYTES into its allocation (multiple of 256): "
                         "moves the streams of one chunk relative to each other in the address space")
    ap.add_argument("--one-arena", action="store_true",
                    help="carve all device chunk lists out of one allocation (list bases 2 MiB-aligned, plus --arena-skew per list)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-wg", default="", metavar="LIST",
                    help="after the timed steps, time the Adam launch with each of these caps on resident workgroups "
                         "per CU (comma list, 0 = no cap), all in the same allocation")
    ap.add_argument("--placements", type=int, default=0, metavar="N",
                    help="after the timed steps, free everything and set the headline workload up again N times "
                         "(alternating chunk reuse off / on), timing the Adam launch in each placement")
    ap.add_argument("--device-state", action="store_true",
                    help="also time the steps with t, the loss scale and the loss-scale bookkeeping on the device (no read-back per step)")
    ap.add_argument("--graph", action="store_true", help="as --device-state, with the step recorded once into a HIP graph and replayed")
    ap.add_argument("--leg", default="", choices=["", "launch_bound", "ragged_packing", "host", "moving_residency"],
                    help="run one leg of the default run alone and print its JSON object (what the default run does in child processes)")
    ap.add_argument("--no-legs", action="store_true",
                    help="default run only: skip the extra legs (chunk reuse on the same workload; the launch-bound tiny "
                         "model; ragged packing; GPT-12.6B with 40 %% of the chunks host-resident, over the link and on the "
                         "host cores; GPT-20B shapes with a moving HBM budget)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also launch psx_copy_bytes once over this many MiB (a plain copy of known size, "
                         "the yardstick the HBM traffic counters are scaled by)")
    ap.add_argument("--fused-unpack", action="store_true",
                    help="write the fp16 parameters to the tensors from inside the Adam launch (psx_chunk_adam_step_unpack) "
                         "instead of a psx_unpack pass that reads the chunks back (all chunks must be HBM-resident)")
    ap.add_argument("--separate-check", action="store_true", help="run the overflow check as a pass of its own (2 B/element more) instead of inside the gradient pack")
    ap.add_argument("--staging-tile", type=int, default=4 << 20, help="elements per staging tile (host-resident chunks)")
    ap.add_argument("--staging-slots", type=int, default=3)
    ap.add_argument("--tune", default="", help="comma list key=value: bpc, unroll, nt, cbpc, threads, wg, cunroll")
    return ap.parse_args()


class State:
    pass


def setup(w, dev, host_fraction=0.0, staging_tile_elems=4 << 20, staging_slots=3, keep_params="all", cpu_share=0.0,
          plans=None, chunk_reuse=False, arena_skew=0, one_arena=False):
    """Allocate chunk lists and seeded inputs on the device (and pinned host memory for
    host-resident chunks); pack the fp32 params tensor by tensor; m = v = 0.
    keep_params: "all" keeps every fp32 source tensor, an int keeps only the first that many, a set keeps
    those indices.
    cpu_share: share of the host-resident chunks that the host cores update (PSX_EXEC_CPU); the rest of
    them is updated by the GPU over the link.
    plans: optional list of per-step residencies (one PSX_LOC_* per chunk); plans[0] is where the fp32
    states start.  A chunk gets a device home if any plan keeps it in HBM and a pinned home if any plan
    puts it on the host.  Without plans the last host_fraction of the chunks live on the host for good."""
    import torch
    from paper_2108_05818_amd import psx
    from paper_2108_05818_amd import workloads as W

    st = State()
    st.w = w
    st.C = w.chunk_elems
    st.slots, st.used = psx.psx_chunk_layout(w.numel, st.C)
    st.nch = len(st.used)
    if plans is None:
        n_host = int(round(host_fraction * st.nch))
        plans = [[psx.PSX_LOC_HBM] * (st.nch - n_host) + [psx.PSX_LOC_HOST] * n_host]
    st.loc = list(plans[0])
    need_dev = [any(pl[k] == psx.PSX_LOC_HBM for pl in plans) for k in range(st.nch)]
    need_host = [any(pl[k] == psx.PSX_LOC_HOST for pl in plans) for k in range(st.nch)]
    n_host = sum(need_host)
    st.n_host = n_host
    n_cpu = int(round(cpu_share * n_host))
    st.n_cpu = n_cpu
    st.ctx = psx.psx_ctx_create(max_chunks=st.nch, max_tensors=len(w.numel),
                                staging_tile_elems=staging_tile_elems if n_host else 0, staging_slots=staging_slots)
    C = st.C

    lists_made = [0]
    pool = {"buf": None, "at": 0}
    if one_arena:
        # every chunk list carved out of ONE device allocation, list bases 2 MiB-aligned plus j*arena_skew
        n_dev = sum(need_dev)
        total = 2 * C * st.nch * (1 if chunk_reuse else 2) + 3 * 4 * C * max(n_dev, 1) + 6 * ((2 << 20) + 8 * max(arena_skew, 0))
        pool["buf"] = torch.zeros(total, dtype=torch.uint8, device=dev)

    def chunk_list(dtype, n):
        """One chunk list = one arena, chunk k at offset k*C (the paper's ChunkLists: a list of chunks per
        tensor type).  Besides being the natural layout it keeps the five streams of a chunk apart in
        memory: p/m/v buffers of one chunk allocated back to back sit at power-of-two distances from each
        other, which costs up to 13 % of the Adam kernel's bandwidth with small chunks."""
        item = torch.empty(0, dtype=dtype).element_size()
        skew = lists_made[0] * arena_skew // item            # elements; list j starts j*arena_skew bytes into its arena
        lists_made[0] += 1
        if pool["buf"] is not None:
            base = (pool["at"] + (2 << 20) - 1) // (2 << 20) * (2 << 20) + skew * item
            nbytes = C * max(n, 1) * item
            arena = pool["buf"][base:base + nbytes].view(dtype)
            pool["at"] = base + nbytes
        else:
            arena = torch.zeros(C * max(n, 1) + skew, dtype=dtype, device=dev)[skew:]
        return [arena[k * C:(k + 1) * C] for k in range(n)]
    st.p16 = chunk_list(torch.float16, st.nch)
    st.g16 = st.p16 if chunk_reuse else chunk_list(torch.float16, st.nch)
    # fp32 states: device homes (one arena per list over the chunks that are ever HBM-resident) and
    # pinned host homes (for the chunks that are ever host-resident)
    p_list, m_list, v_list = (iter(chunk_list(torch.float32, sum(need_dev))) for _ in range(3))
    st.p32, st.m, st.v, st.host = [], [], [], []
    for k in range(st.nch):
        st.p32.append(next(p_list) if need_dev[k] else None)
        st.m.append(next(m_list) if need_dev[k] else None)
        st.v.append(next(v_list) if need_dev[k] else None)
        # a host-resident chunk needs room for its used prefix only (pinned memory is scarce)
        st.host.append([psx.PinnedF32(st.used[k]) for _ in range(3)] if need_host[k] else None)
    # seeded tensors (the "model"): fp32 params, packed one tensor at a time straight into the chunk
    # that will hold them (pinned host chunks are device-accessible, so the pack kernel writes them too),
    # and one set of scaled fp16 gradients
    p32_dst = psx.ptr_array([st.p32[k] if st.loc[k] == psx.PSX_LOC_HBM else st.host[k][0] for k in range(st.nch)])
    st.p_t = []
    for i, s in enumerate(w.numel):
        t = W.params_torch(s, w.seed + i, dev)
        one = (psx.psx_slot * 1)(st.slots[i])
        lib_chunks = p32_dst
        psx.lib().psx_pack(st.ctx, psx.PSX_F32, psx.ptr_array([t]), one, 1, lib_chunks, st.nch, C, 0,
                           torch.cuda.current_stream().cuda_stream)
        keep = keep_params == "all" or (i in keep_params if isinstance(keep_params, (set, frozenset)) else i < keep_params)
        st.p_t.append(t if keep else None)
    torch.cuda.synchronize()
    st.g_t = [W.grads_f16_torch(s, w.seed + 100000 + i, w.loss_scale, dev) for i, s in enumerate(w.numel)]
    st.out_t = [torch.empty(s, dtype=torch.float16, device=dev) for s in w.numel]
    st.specs = []
    for k in range(st.nch):
        s = dict(g16=st.g16[k], p16=st.p16[k], used=st.used[k], loc_in=st.loc[k], loc_out=st.loc[k])
        if need_dev[k]:
            s.update(p32=st.p32[k], m=st.m[k], v=st.v[k])
        if need_host[k]:
            s.update(p32_host=st.host[k][0], m_host=st.host[k][1], v_host=st.host[k][2],
                     exec=psx.PSX_EXEC_CPU if k >= st.nch - n_cpu else psx.PSX_EXEC_GPU)
        st.specs.append(s)
    st.chunks = psx.make_chunks(st.specs)
    st.t_ptrs = psx.ptr_array(st.g_t)
    st.o_ptrs = psx.ptr_array(st.out_t)
    st.scaler = psx.make_scaler(w.loss_scale, w.growth_interval)
    st.numel_arr = list(w.numel)
    st.numel_c = (ctypes.c_uint64 * max(len(w.numel), 1))(*w.numel)
    st.slots_c = (psx.psx_slot * max(len(w.numel), 1))()
    st.used_c = (ctypes.c_uint64 * st.nch)()
    return st


def run_step(st, fused_check=False, new_loc=None, fused_unpack=False):
    """One pass of the hot path; returns the overflow flag.  new_loc: where each chunk's fp32 states are
    to live after this step (default: where they are)."""
    from paper_2108_05818_amd import psx
    w, ctx, C = st.w, st.ctx, st.C
    if new_loc is not None and list(new_loc) != st.loc:
        for k, s in enumerate(st.specs):
            s["loc_in"], s["loc_out"] = st.loc[k], new_loc[k]
        st.chunks = psx.make_chunks(st.specs)
        st.loc, st.settled = list(new_loc), False
    elif not getattr(st, "settled", True):          # the chunks that moved last step now stay where they are
        for k, s in enumerate(st.specs):
            s["loc_in"] = s["loc_out"] = st.loc[k]
        st.chunks = psx.make_chunks(st.specs)
        st.settled = True
    # a1: the layout call itself, into arrays marshalled once (building ctypes arrays of thousands of
    # tensor sizes every step is Python overhead, not the call)
    nch_out = ctypes.c_size_t(0)
    rc = psx.lib().psx_chunk_layout(st.numel_c, len(st.numel_arr), C, 0, st.slots_c, st.used_c, st.nch,
                                    ctypes.byref(nch_out))
    if rc != 0 or nch_out.value != st.nch:
        raise RuntimeError(f"psx_chunk_layout: {rc} {psx.psx_last_error()}")
    slots = st.slots_c
    n = len(st.numel_arr)
    if fused_check:
        psx.psx_overflow_reset(ctx)
        psx.psx_pack(ctx, psx.PSX_F16, st.t_ptrs, slots, st.g16, C, flags=psx.PSX_PACK_CHECK_OVERFLOW, n=n)   # a2 + a3
        step_flags = psx.PSX_STEP_USE_FLAG
    else:
        psx.psx_pack(ctx, psx.PSX_F16, st.t_ptrs, slots, st.g16, C, n=n)     # a2
        step_flags = psx.PSX_STEP_CHECK_FIRST                                 # a3 inside the step call
    hp = psx.make_hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                        adamw_mode=w.adamw_mode, step=st.scaler.step, loss_scale=st.scaler.scale)
    if fused_unpack:                                                           # a4 / a6 with a2's unpack inside the launch
        psx.psx_chunk_adam_step_unpack(ctx, st.chunks, hp, step_flags, st.o_ptrs, slots, C, n_chunks=st.nch, n=n)
    else:
        psx.psx_chunk_adam_step(ctx, st.chunks, hp, step_flags, n_chunks=st.nch)  # a4 / a5 / a6
        psx.psx_unpack(ctx, psx.PSX_F16, st.o_ptrs, slots, st.p16, C, n=n)       # a2 (fp16 params back to tensors)
    flag, _ = psx.psx_overflow_read(ctx)                                      # synchronises the stream
    psx.psx_loss_scale_update(st.scaler, flag)                                # a7
    return flag


def step_on_device(st, lean=False):
    """One pass of the hot path with nothing read back: the update takes t and the loss scale from the
    context's step state on the device and the loss-scale bookkeeping (a7) runs there too.  Kernel
    launches only once the descriptor tables are on the device, so it can be recorded into a HIP graph.
    lean: the same work in three launches instead of five: the fp16 unpack inside the update and the
    flags cleared by the bookkeeping kernel of the step before (the caller clears them once at the start)."""
    from paper_2108_05818_amd import psx
    ctx, C, n = st.ctx, st.C, len(st.numel_arr)
    if lean:
        psx.psx_pack(ctx, psx.PSX_F16, st.t_ptrs, st.slots_c, st.g16, C, flags=psx.PSX_PACK_CHECK_OVERFLOW, n=n)
        psx.psx_chunk_adam_step_unpack(ctx, st.chunks, st.hyper_dev, psx.PSX_STEP_USE_FLAG | psx.PSX_STEP_DEVICE_STATE,
                                       st.o_ptrs, st.slots_c, C, n_chunks=st.nch, n=n)
        psx.psx_step_state_advance(ctx, psx.PSX_ADVANCE_CLEAR_FLAGS)
        return
    psx.psx_overflow_reset(ctx)
    psx.psx_pack(ctx, psx.PSX_F16, st.t_ptrs, st.slots_c, st.g16, C, flags=psx.PSX_PACK_CHECK_OVERFLOW, n=n)
    psx.psx_chunk_adam_step(ctx, st.chunks, st.hyper_dev, psx.PSX_STEP_USE_FLAG | psx.PSX_STEP_DEVICE_STATE, n_chunks=st.nch)
    psx.psx_unpack(ctx, psx.PSX_F16, st.o_ptrs, st.slots_c, st.p16, C, n=n)
    psx.psx_step_state_advance(ctx)


def timed_steps_on_device(st, steps, warmup, graph, lean=False):
    """Steps that never synchronise (step state on the device), eagerly enqueued or as replays of one HIP
    graph; the layout call (host) is still made every step.  Returns wall ms per step and the state read
    back at the end."""
    import torch
    from paper_2108_05818_amd import psx
    w = st.w
    st.hyper_dev = psx.make_hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                                  adamw_mode=w.adamw_mode)
    psx.psx_ctx_set_profiling(st.ctx, 0)
    psx.psx_step_state_init(st.ctx, st.hyper_dev, st.scaler)
    nch_out = ctypes.c_size_t(0)

    def layout():
        rc = psx.lib().psx_chunk_layout(st.numel_c, len(st.numel_arr), st.C, 0, st.slots_c, st.used_c, st.nch, ctypes.byref(nch_out))
        if rc != 0:
            raise RuntimeError(psx.psx_last_error())
    layout()
    psx.psx_overflow_reset(st.ctx)
    for _ in range(max(warmup, 1)):            # also uploads the descriptor tables the recorded calls rely on
        layout(); step_on_device(st, lean)
    torch.cuda.synchronize()
    g = None
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step_on_device(st, lean)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        layout()
        if g is not None:
            g.replay()
        else:
            step_on_device(st, lean)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / max(steps, 1)
    sc, last_flag, skipped = psx.psx_step_state_read(st.ctx)
    return {"ms": ms, "step": int(sc.step), "scale": float(sc.scale), "skipped": int(skipped)}


def leg_launch_bound(dev):
    """The tiny GPT (3 chunks, 0.17 M elements), where launches and the flag read-back are the step: with the
    host in the loop, with the step state on the device, and as replays of one HIP graph."""
    from paper_2108_05818_amd import workloads as W
    w = W.config1_tiny()
    out = {"workload": w.name, "n_elems": w.n_elems, "steps": 500, "warmup": 20}
    st = setup(w, dev, keep_params=0)
    out["host_bookkeeping_us_per_step"] = timed_steps(st, 500, 20, True)["ms"] * 1e3
    release(st)
    for key, graph, lean in (("device_state_us_per_step", False, False), ("graph_replay_us_per_step", True, False),
                             ("graph_replay_three_launches_us_per_step", True, True)):
        st = setup(w, dev, keep_params=0)
        r = timed_steps_on_device(st, 500, 20, graph, lean)
        assert r["skipped"] == 0 and r["step"] == 1 + 500 + 20 + (0 if not graph else 0), r
        out[key] = r["ms"] * 1e3
        release(st)
    return out


def cpu_baseline(st, target_chunks=16):
    """The oracle, as it stands, on the host cores: one whole step (gradient pack, overflow check,
    Adam, fp16 unpack) over the first tensors of the workload that fill `target_chunks` chunks, with
    tensors and chunks spread over threads (the oracle's own code is single-threaded C); then the same
    step on one thread over the first tensors that fill at least one chunk (the parity reference as
    the tests run it)."""
    import numpy as np
    import torch
    import oracle as orc

    w, C = st.w, st.C
    o_slots, o_used = orc.chunk_layout(w.numel, C)

    def prefix(chunks_wanted, at_least_one_chunk=False):
        """Tensors 0..T-1: the longest prefix that ends inside the first `chunks_wanted` chunks
        (or, with at_least_one_chunk, the shortest one that fills a whole chunk)."""
        T = 0
        for i in range(min(len(w.numel), CPU_BASELINE_TENSORS)):
            end = o_slots[i].chunk * C + o_slots[i].offset + o_slots[i].numel
            if at_least_one_chunk:
                T = i + 1
                if end >= C:
                    break
            else:
                if end > chunks_wanted * C:
                    break
                T = i + 1
        return max(T, 1)

    def one_step(T, threads):
        numel = w.numel[:T]
        slots, used = orc.chunk_layout(numel, C)
        nch = len(used)
        n_elems = int(sum(numel))
        threads = max(1, min(threads, max(nch, 1)))
        g_np = [st.g_t[i].view(torch.int16).cpu().numpy().view(np.uint16) for i in range(T)]
        p_np = [st.p_t[i].cpu().numpy() for i in range(T)]
        ch = dict(p32=[np.zeros(C, np.float32) for _ in range(nch)], m=[np.zeros(C, np.float32) for _ in range(nch)],
                  v=[np.zeros(C, np.float32) for _ in range(nch)], p16=[np.zeros(C, np.uint16) for _ in range(nch)],
                  g16=[np.zeros(C, np.uint16) for _ in range(nch)])
        out = [np.zeros(s, np.uint16) for s in numel]
        sub = lambda i: (orc.Slot * 1)(slots[i])
        pool = ThreadPoolExecutor(threads)
        list(pool.map(lambda i: orc.pack([p_np[i]], sub(i), ch["p32"], C), range(T)))          # untimed set-up
        h = orc.hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                      adamw_mode=w.adamw_mode, step=1, loss_scale=w.loss_scale)
        t0 = time.perf_counter()
        orc.chunk_layout(numel, C)
        list(pool.map(lambda i: orc.pack([g_np[i]], sub(i), ch["g16"], C), range(T)))
        flags = list(pool.map(lambda k: orc.overflow_check([ch["g16"][k]], [used[k]])[0], range(nch)))
        if not any(flags):
            list(pool.map(lambda k: orc.adam_chunk(ch["g16"][k], ch["p16"][k], ch["p32"][k], ch["m"][k], ch["v"][k],
                                                   int(used[k]), h), range(nch)))
        list(pool.map(lambda i: orc.unpack([out[i]], sub(i), ch["p16"], C), range(T)))
        dt = time.perf_counter() - t0
        pool.shutdown()
        return n_elems, nch, threads, dt, T

    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    n_elems, nch, threads, dt, T = one_step(prefix(target_chunks), cores)
    n1, nch1, _, dt1, T1 = one_step(prefix(1, at_least_one_chunk=True), 1)
    return {"value": n_elems / dt / 1e9, "unit": "Gelem/s", "cores": threads, "kind": "oracle",
            "sample": f"one whole step on the first {T} tensors ({n_elems} elements, {nch} chunks of {C}) "
                      f"of the same workload, {dt:.2f} s wall on {threads} threads",
            "single_thread": {"value": n1 / dt1 / 1e9, "unit": "Gelem/s", "cores": 1,
                              "sample": f"the same step on the first {T1} tensor(s) ({n1} elements, {nch1} chunks of {C}), "
                                        f"{dt1:.2f} s wall on one thread"}}


def read_traffic(path):
    """HBM bytes per Adam launch from the committed counter summary (None if absent)."""
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


def pick_workload(a):
    """-> (workload, host_fraction, plans, scaled_from)."""
    from paper_2108_05818_amd import psx
    from paper_2108_05818_amd import workloads as W
    scaled_from = None
    if a.workload == "tiny":
        w = W.config1_tiny()
    elif a.workload == "ragged":
        w = W.config3_ragged()
    elif a.workload == "gpt12b":
        w = W.config4_gpt12b(a.layers or 40)
        if w.name != W.config4_gpt12b().name:
            scaled_from = f"{W.config4_gpt12b().name}: layer count only; hidden size, vocabulary and chunk size kept"
    elif a.workload == "gpt20b":
        # 44 layers need 170 GB of pinned memory; 12 layers of the same tensors fit this box's limit
        w = W.config5_gpt20b(a.layers or 12)
        if w.name != W.config5_gpt20b().name:
            scaled_from = (f"{W.config5_gpt20b().name} (401 chunks, about 170 GB of pinned host state; the box pins at most "
                           "65 GiB): layer count only; hidden size, vocabulary and chunk size kept")
    else:
        w = W.config2_gpt1b(a.layers or 20)
        if w.name != W.config2_gpt1b().name:
            scaled_from = f"{W.config2_gpt1b().name}: layer count only"
    if a.chunk_elems:
        w.chunk_elems = a.chunk_elems
        w.name += f"-C{a.chunk_elems}"
    host_fraction = w.host_fraction if a.host_fraction < 0 else a.host_fraction
    plans = None
    if a.workload == "gpt20b":
        # the HBM budget for fp32 states moves by +-30 % from step to step (seeded); the planner keeps the
        # fullest chunks that fit, the rest live in pinned host memory; chunks at the margin change residence
        # while they are updated
        _, used = psx.psx_chunk_layout(w.numel, w.chunk_elems)
        per_chunk = 12 * w.chunk_elems
        budget = lambda t: int(round(len(used) * W.budget_fraction(t, 1.0 - host_fraction, w.budget_jitter, w.seed))) * per_chunk
        plans = [psx.psx_plan_residency(used, w.chunk_elems, budget(t))[0] for t in range(a.warmup + a.steps + 1)]
    return w, host_fraction, plans, scaled_from


def timed_steps(st, steps, warmup, fused_check, plans=None, fused_unpack=False):
    """`warmup` untimed steps, then exactly `steps` timed ones between two device synchronisations.
    Returns wall ms per step, the per-launch HIP-event times averaged over the timed steps, the link
    bytes summed over them, and the last step's psx_timing."""
    import torch
    from paper_2108_05818_amd import psx
    psx.psx_ctx_set_profiling(st.ctx, 1)
    plan_at = (lambda t: plans[t]) if plans else (lambda t: None)
    for i in range(warmup):
        run_step(st, fused_check, plan_at(1 + i), fused_unpack)
    torch.cuda.synchronize()
    phase = {"pack_ms": 0.0, "check_ms": 0.0, "adam_ms": 0.0, "unpack_ms": 0.0, "spill_ms": 0.0}
    link = {"h2d": 0, "d2h": 0, "min_h2d": 0, "min_d2h": 0, "moved_chunks": 0, "resident_chunks": []}
    skipped = 0
    tm = None
    each_step, each_adam = [], []
    t0 = time.perf_counter()
    for i in range(steps):
        before = list(st.loc)
        ts = time.perf_counter()
        skipped += run_step(st, fused_check, plan_at(1 + warmup + i), fused_unpack)
        each_step.append((time.perf_counter() - ts) * 1e3)   # the step ends with the flag read back: the stream is drained
        tm = psx.psx_ctx_get_timing(st.ctx)      # events of this step
        each_adam.append(tm.adam_ms)
        phase["pack_ms"] += tm.pack_ms; phase["check_ms"] += tm.check_ms; phase["unpack_ms"] += tm.unpack_ms
        phase["adam_ms"] += tm.adam_ms; phase["spill_ms"] += tm.spill_ms
        # every chunk that starts the step on the host must come in once, every chunk that ends it there
        # must go out once: 12 bytes per used element each
        link["h2d"] += int(tm.h2d_bytes); link["d2h"] += int(tm.d2h_bytes)
        link["min_h2d"] += 12 * sum(u for u, l, s in zip(st.used, before, st.specs) if l == psx.PSX_LOC_HOST and s.get("exec", 0) == psx.PSX_EXEC_GPU)
        link["min_d2h"] += 12 * sum(u for u, l, s in zip(st.used, st.loc, st.specs) if l == psx.PSX_LOC_HOST and s.get("exec", 0) == psx.PSX_EXEC_GPU)
        link["moved_chunks"] += sum(x != y for x, y in zip(before, st.loc))
        link["resident_chunks"].append(sum(l == psx.PSX_LOC_HBM for l in st.loc))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sums = dict(phase)
    for k in phase:
        phase[k] /= max(steps, 1)
    return {"ms": dt * 1e3 / max(steps, 1), "phase": phase, "phase_sum_ms": sums, "link": link, "tm": tm, "skipped": skipped,
            "step_ms": spread(each_step), "adam_launch_ms": spread(each_adam)}


def spread(xs):
    """Median, minimum and maximum of per-step times."""
    if not xs:
        return None
    xs = sorted(xs)
    mid = len(xs) // 2
    med = xs[mid] if len(xs) % 2 else 0.5 * (xs[mid - 1] + xs[mid])
    return {"median": med, "min": xs[0], "max": xs[-1]}


def plain_copy_rate(ctx, dev):
    """A same-run yardstick for the roofline: this library's plain copy kernel over 1 GiB (1 read + 1 write stream)."""
    import torch
    from paper_2108_05818_amd import psx
    nb = 1 << 30
    src = torch.ones(nb // 4, dtype=torch.float32, device=dev)
    dst = torch.zeros_like(src)
    for _ in range(3):
        psx.psx_copy_bytes(ctx, dst, src, nb)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        psx.psx_copy_bytes(ctx, dst, src, nb)         # launched on torch's current stream, as the events are
    e1.record()
    torch.cuda.synchronize()
    return 10 * 2 * nb / (e0.elapsed_time(e1) * 1e-3) / 1e9


def adam_roofline(r, copy_gbs=None, bytes_per_elem=ADAM_BYTES_PER_ELEM):
    """HBM roofline of the resident Adam launch from the HIP-event times of `timed_steps`."""
    adam_elems = int(r["tm"].adam_elems)
    adam_bytes = bytes_per_elem * adam_elems
    ms = r["phase"]["adam_ms"]
    achieved = adam_bytes / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
    out = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
           "kernel": ("psx::adam_out_kernel (resident chunks and the fp16 tensors, one launch)" if bytes_per_elem != ADAM_BYTES_PER_ELEM
                      else "psx::adam_kernel (resident chunks, one launch)"),
           "bytes_per_launch": adam_bytes, "avg_launch_ms": ms,
           "launch_ms": r.get("adam_launch_ms")}
    if copy_gbs:
        out.update(same_run_plain_copy_GBs=copy_gbs, frac_of_plain_copy=achieved / copy_gbs)
    return out


def host_link_report(st, r, mode):
    """Achieved link rates of the host-resident part over the timed steps (bytes and span times summed
    over all of them), next to both same-run pinned-copy rates of this machine."""
    from paper_2108_05818_amd import psx
    tm, link = r["tm"], r["link"]
    link_s = r["phase_sum_ms"]["spill_ms"] * 1e-3
    rates = psx.psx_measure_link(st.ctx, 1024, 5)      # same copy streams as the staged pipeline, pinned memory
    peak = {"copy_h2d_alone_GBs": rates.h2d_alone, "copy_d2h_alone_GBs": rates.d2h_alone,
            "copy_each_way_both_at_once_GBs": rates.each_way_both, "copy_MiB": 1024}
    h2d = link["h2d"] / link_s / 1e9 if link_s and link["h2d"] else None
    d2h = link["d2h"] / link_s / 1e9 if link_s and link["d2h"] else None
    each = min(x for x in (h2d, d2h) if x) if (h2d or d2h) else None
    steps = max(len(link["resident_chunks"]), 1)
    return {"bound": "host link, 12 B/element each way, both directions at once",
            "mode": {1: "direct (the kernel reads and writes pinned memory over the link)", 0: "staged (H2D, kernel, D2H on copy streams)"}[mode],
            "h2d_GBs": h2d, "d2h_GBs": d2h, "measured_peak": peak,
            # two denominators: the best pinned-copy rate of one direction alone, and what hipMemcpyAsync
            # reaches per direction with both directions busy (less, with this runtime)
            "frac": each / max(rates.h2d_alone, rates.d2h_alone) if each else None,
            "frac_of_copies_both_at_once": each / rates.each_way_both if each else None,
            "host_cores": {"elems": int(tm.cpu_elems), "threads": int(tm.cpu_threads), "ms": float(tm.cpu_ms),
                           "gelem_s": tm.cpu_elems / (tm.cpu_ms * 1e-3) / 1e9 if tm.cpu_ms else None},
            "host_part_gelem_s": (tm.spill_elems + tm.cpu_elems) * steps / link_s / 1e9 if link_s else None,
            "spill_elems": int(tm.spill_elems), "spill_ms": r["phase"]["spill_ms"],
            "link_bytes": link["h2d"] + link["d2h"], "link_bytes_minimum": link["min_h2d"] + link["min_d2h"]}


def release(st):
    import gc
    import torch
    from paper_2108_05818_amd import psx
    psx.psx_ctx_destroy(st.ctx)
    for hs in st.host:
        for b in hs or []:
            b.free()
    st.__dict__.clear()
    gc.collect()
    torch.cuda.empty_cache()


def leg_chunk_reuse(st):
    """The paper's layout (Sec. "Preprocessing Stage": the gradient sits in the param fp16 chunk) on the
    headline workload and on the headline's own buffers: the gradient list is dropped and gradients are
    packed into the fp16 parameter chunks, so the Adam launch reads gradients from, and writes parameters
    to, the same fp16 chunk.  Same p32/m/v/p16 memory as the headline: only the aliasing differs."""
    from paper_2108_05818_amd import psx
    w = st.w
    for k, s in enumerate(st.specs):
        s["g16"] = st.p16[k]
    st.g16 = st.p16
    st.chunks = psx.make_chunks(st.specs)
    r = timed_steps(st, 10, 3, True)
    return {"workload": w.name, "steps": 10, "warmup": 3, "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9,
            "bytes_of_chunk_lists_per_param": 14, "roofline": adam_roofline(r)}


def leg_views(st, steps=10, warmup=3):
    """The paper's own arrangement on the headline's buffers: tensors are views into the chunk lists, so nothing
    is packed or unpacked (row a2 does not occur); a step is the overflow test over the gradient chunks, the
    update, the flag read-back and the loss-scale bookkeeping: 2 + 28 bytes per element."""
    import torch
    from paper_2108_05818_amd import psx
    w = st.w
    psx.psx_ctx_set_profiling(st.ctx, 1)

    def step():
        hp = psx.make_hyper(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay,
                            adamw_mode=w.adamw_mode, step=st.scaler.step, loss_scale=st.scaler.scale)
        psx.psx_chunk_adam_step(st.ctx, st.chunks, hp, psx.PSX_STEP_CHECK_FIRST, n_chunks=st.nch)
        flag, _ = psx.psx_overflow_read(st.ctx)
        psx.psx_loss_scale_update(st.scaler, flag)
        return flag
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    adam_ms = check_ms = 0.0
    skipped = 0
    t0 = time.perf_counter()
    for _ in range(steps):
        skipped += step()
        tm = psx.psx_ctx_get_timing(st.ctx)
        adam_ms += tm.adam_ms; check_ms += tm.check_ms
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return {"workload": w.name, "steps": steps, "warmup": warmup, "ms_per_step": ms, "gelem_s": w.n_elems / (ms * 1e-3) / 1e9,
            "bytes_per_elem_of_the_step": 30, "check_ms": check_ms / steps, "adam_ms": adam_ms / steps, "skipped_steps": skipped}


def leg_fused_unpack(st):
    """The headline step on the headline's own buffers with the fp16 parameters written to the tensors from
    inside the Adam launch (psx_chunk_adam_step_unpack) instead of a psx_unpack pass that reads the chunks
    back: 4 + 30 bytes per element in two launches instead of 4 + 28 + 4 in three."""
    w = st.w
    r = timed_steps(st, 10, 3, True, fused_unpack=True)
    inside = r["phase"]["unpack_ms"] == 0           # else the library chose two launches (tensors not aligned like their slots)
    return {"workload": w.name, "steps": 10, "warmup": 3, "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9,
            "bytes_per_elem_of_the_step": 34 if inside else 36, "phase_ms": r["phase"],
            "roofline": adam_roofline(r, bytes_per_elem=ADAM_BYTES_PER_ELEM + (2 if inside else 0))}


def placement_trials(a, dev, n):
    """The Adam launch time over n fresh set-ups of the headline workload in this process, alternating a
    gradient list of its own with chunk reuse.  Every set-up frees and re-allocates all buffers, so the
    virtual addresses repeat while the physical placement changes: what varies between trials of one
    kind is where the chunk lists landed in HBM."""
    from paper_2108_05818_amd import workloads as W
    out = []
    for t in range(n):
        w = W.config2_gpt1b()
        st = setup(w, dev, keep_params=0, chunk_reuse=bool(t % 2), arena_skew=a.arena_skew, one_arena=a.one_arena)
        r = timed_steps(st, 8, 3, True)
        out.append({"trial": t, "chunk_reuse": bool(t % 2), "adam_ms": r["phase"]["adam_ms"], "frac": adam_roofline(r)["frac"]})
        release(st)
    return out


def sweep_wg(st, values):
    """Adam launch time against the cap on resident workgroups per CU, in one allocation (so the
    placement of the buffers in memory is the same for every value)."""
    from paper_2108_05818_amd import psx
    out = {}
    for wg in values:
        psx.psx_ctx_set_tuning(st.ctx, psx.PSX_TUNE_ADAM_WG_PER_CU, wg)
        r = timed_steps(st, 3, 1, True)
        out[str(wg)] = {"adam_ms": r["phase"]["adam_ms"], "frac": adam_roofline(r)["frac"]}
    psx.psx_ctx_set_tuning(st.ctx, psx.PSX_TUNE_ADAM_WG_PER_CU, 14)
    return out


def leg_host(a, dev):
    """Config 4 at full size (GPT-12.6B, 244 chunks of 64 Mi, the last 40 % host-resident), first with the
    GPU updating the host-resident chunks over the link (the benchmark spec's spilled case), then with the host
    cores updating them (the paper's own placement for host-resident optimizer states)."""
    from paper_2108_05818_amd import psx
    from paper_2108_05818_amd import workloads as W
    w = W.config4_gpt12b()
    st = setup(w, dev, w.host_fraction, a.staging_tile, a.staging_slots, keep_params=0)
    mode = 1
    r = timed_steps(st, 5, 2, True)
    link = {"workload": w.name, "n_elems": w.n_elems, "n_chunks": st.nch, "host_resident_chunks": st.n_host,
            "steps": 5, "warmup": 2, "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9,
            "resident_adam_ms": r["phase"]["adam_ms"]}
    link.update(host_link_report(st, r, mode))
    cores = None
    if psx_cpu_ok():
        for s in st.specs:
            if s.get("loc_in") == psx.PSX_LOC_HOST:
                s["exec"] = psx.PSX_EXEC_CPU
        st.chunks = psx.make_chunks(st.specs)
        r = timed_steps(st, 3, 1, True)
        tm = r["tm"]
        cores = {"workload": w.name, "steps": 3, "warmup": 1, "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9,
                 "host_elems": int(tm.cpu_elems), "threads": int(tm.cpu_threads), "host_update_ms": float(tm.cpu_ms),
                 "host_gelem_s": tm.cpu_elems / (tm.cpu_ms * 1e-3) / 1e9 if tm.cpu_ms else None,
                 "host_dram_GBs": ADAM_BYTES_PER_ELEM * tm.cpu_elems / (tm.cpu_ms * 1e-3) / 1e9 if tm.cpu_ms else None,
                 "link_bytes_per_elem": 4, "resident_adam_ms": r["phase"]["adam_ms"]}
    release(st)
    return link, cores


def residency_report(r, w, host_fraction):
    link = r["link"]
    moved = link["h2d"] + link["d2h"]
    floor = link["min_h2d"] + link["min_d2h"]
    return {"hbm_budget": f"{1.0 - host_fraction:.2f} of the fp32-state chunks, x (1 + {w.budget_jitter} u_t), u_t ~ U(-1, 1) seeded",
            "resident_chunks_per_step": link["resident_chunks"], "chunks_that_changed_residence": link["moved_chunks"],
            "link_bytes": moved, "link_bytes_minimum": floor, "link_bytes_over_minimum": moved / floor if floor else None}


def leg_ragged(dev):
    """Config 3: 5000 tensors with log-uniform sizes in 16 Mi chunks; what it stresses is the multi-tensor pack and
    unpack (segments with arbitrary alignment), the Adam launch is the headline's kernel on another chunk size."""
    from paper_2108_05818_amd import workloads as W
    w = W.config3_ragged()
    st = setup(w, dev, keep_params=0)
    r = timed_steps(st, 10, 3, True)
    out = {"workload": w.name, "n_elems": w.n_elems, "n_tensors": len(w.numel), "n_chunks": st.nch, "chunk_elems": w.chunk_elems,
           "steps": 10, "warmup": 3, "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9,
           "pack_ms": r["phase"]["pack_ms"], "pack_GBs": 4 * w.n_elems / (r["phase"]["pack_ms"] * 1e-3) / 1e9,
           "unpack_ms": r["phase"]["unpack_ms"], "unpack_GBs": 4 * w.n_elems / (r["phase"]["unpack_ms"] * 1e-3) / 1e9,
           "roofline": adam_roofline(r)}
    release(st)
    return out


def leg_moving_residency(a, dev):
    """Config 5's tensor shapes at 12 layers: the HBM budget moves by +-30 % per step (seeded), psx_plan_residency
    picks each step's resident set, chunks at its margin change residence while they are updated."""
    import argparse as _ap
    b = _ap.Namespace(**vars(a))
    b.workload, b.layers, b.chunk_elems, b.host_fraction, b.steps, b.warmup = "gpt20b", 0, 0, -1.0, 6, 2
    w, host_fraction, plans, scaled_from = pick_workload(b)
    st = setup(w, dev, host_fraction, a.staging_tile, a.staging_slots, keep_params=0, plans=plans)
    r = timed_steps(st, b.steps, b.warmup, True, plans)
    out = {"workload": w.name, "scaled_from": scaled_from, "n_elems": w.n_elems, "n_chunks": st.nch, "steps": b.steps, "warmup": b.warmup,
           "ms_per_step": r["ms"], "gelem_s": w.n_elems / (r["ms"] * 1e-3) / 1e9}
    hl = host_link_report(st, r, 1)
    out.update({k: hl[k] for k in ("h2d_GBs", "d2h_GBs", "frac", "frac_of_copies_both_at_once")})
    out["residency"] = residency_report(r, w, host_fraction)
    release(st)
    return out


def run_leg(name):
    """Run one leg as a child process (`bench.py --leg NAME`) and return the JSON object it prints."""
    import subprocess
    try:
        r = subprocess.run([sys.executable, os.path.abspath(__file__), "--leg", name], capture_output=True, text=True, timeout=400)
        lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
        if r.returncode != 0 or not lines:
            return {"error": f"leg {name}: exit status {r.returncode}: {r.stderr.strip()[-400:]}"}
        return json.loads(lines[-1])
    except subprocess.TimeoutExpired:
        return {"error": f"leg {name}: no result within 400 s"}


def psx_cpu_ok():
    """PSX_EXEC_CPU needs AVX2 + F16C on the host."""
    try:
        flags = open("/proc/cpuinfo").read()
        return " avx2" in flags and " f16c" in flags
    except OSError:
        return False


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this path has no collectives and is not sharded here; "
              "run with --gpus 1 (total throughput of N GPUs is N independent copies of this number).",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2108_05818_amd import psx

    if not os.path.exists(psx.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    if a.leg:
        if a.leg == "launch_bound":
            res = leg_launch_bound(dev)
        elif a.leg == "ragged_packing":
            res = leg_ragged(dev)
        elif a.leg == "host":
            link, cores = leg_host(a, dev)
            res = {"host_link": link, "host_cores": cores}
        else:
            res = leg_moving_residency(a, dev)
        print(json.dumps(res))
        return
    w, host_fraction, plans, scaled_from = pick_workload(a)
    # the default run (headline workload, no overrides) appends the other halves of the metric as legs
    headline = (a.workload == "gpt1b" and not a.layers and not a.chunk_elems and host_fraction == 0
                and not a.chunk_reuse and not a.tune and not a.arena_skew and not a.one_arena and not a.fused_unpack)
    legs = headline and not a.no_legs
    # the fp32 source tensors are needed again only by the oracle leg, and only the first few of them
    st = setup(w, dev, host_fraction, a.staging_tile, a.staging_slots,
               keep_params=0 if a.no_cpu_baseline else CPU_BASELINE_TENSORS,
               cpu_share=0.0 if plans else a.cpu_share, plans=plans, chunk_reuse=a.chunk_reuse,
               arena_skew=a.arena_skew, one_arena=a.one_arena)
    tune_keys = {"bpc": psx.PSX_TUNE_ADAM_BLOCKS_PER_CU, "unroll": psx.PSX_TUNE_ADAM_UNROLL,
                 "nt": psx.PSX_TUNE_NONTEMPORAL, "cbpc": psx.PSX_TUNE_COPY_BLOCKS_PER_CU,
                 "threads": psx.PSX_TUNE_ADAM_THREADS, "wg": psx.PSX_TUNE_ADAM_WG_PER_CU,
                 "cunroll": psx.PSX_TUNE_COPY_UNROLL, "hostmode": psx.PSX_TUNE_HOST_MODE,
                 "hostgrid": psx.PSX_TUNE_HOST_GRID, "hostunroll": psx.PSX_TUNE_HOST_UNROLL,
                 "cputhreads": psx.PSX_TUNE_CPU_THREADS, "cputile": psx.PSX_TUNE_CPU_TILE_ELEMS,
                 "cpuisa": psx.PSX_TUNE_CPU_ISA, "cthreads": psx.PSX_TUNE_COPY_THREADS}
    host_mode = 1
    for kv in filter(None, a.tune.split(",")):
        k, v = kv.split("=")
        psx.psx_ctx_set_tuning(st.ctx, tune_keys[k], int(v))
        if k == "hostmode":
            host_mode = int(v)

    if a.copy_calibration:
        nb = a.copy_calibration << 20
        src = torch.ones(nb // 4, dtype=torch.float32, device=dev)
        dst = torch.zeros_like(src)
        psx.psx_copy_bytes(st.ctx, dst, src, nb)
        torch.cuda.synchronize()
        del src, dst
    cpu = None
    if not a.no_cpu_baseline:
        cpu = cpu_baseline(st)

    r = timed_steps(st, a.steps, a.warmup, not a.separate_check, plans, a.fused_unpack)
    ms, phase, tm = r["ms"], r["phase"], r["tm"]
    on_device = None
    if a.device_state or a.graph:
        # the same workload once more with the step state on the device (--graph: as replays of one HIP graph)
        rd = timed_steps_on_device(st, a.steps, a.warmup, a.graph)
        on_device = {"mode": "graph replay" if a.graph else "eager, no read-back", "ms_per_step": rd["ms"],
                     "gelem_s": w.n_elems / (rd["ms"] * 1e-3) / 1e9, "steps_skipped": rd["skipped"]}
    n_elems = w.n_elems
    copy_gbs = plain_copy_rate(st.ctx, dev)
    # with the unpack fused in, the launch also writes the fp16 parameters to the tensors: 2 B/element more
    # (the library runs update and unpack as two launches of its own when the tensors are not aligned like their
    # slots: then the timings show an unpack launch and the Adam launch is the 28-byte one)
    wrote_tensors = a.fused_unpack and r["phase"]["unpack_ms"] == 0
    roofline = adam_roofline(r, copy_gbs, ADAM_BYTES_PER_ELEM + (2 if wrote_tensors else 0))
    traffic_file = os.path.join("profiles", "adam_kernel_gpt1b_hbm_traffic.txt")
    roofline["traffic"] = read_traffic(os.path.join(ROOT, traffic_file)) if headline else None
    # not a quantity of this run: HBM bytes per launch from the committed FETCH_SIZE / WRITE_SIZE counter runs
    roofline["traffic_source"] = traffic_file if roofline["traffic"] is not None else None
    adam_elems = int(tm.adam_elems)
    out = {
        "metric": "chunked Adam Gelem/s (whole hot path per step: layout + grad pack + overflow check + fused Adam + fp16 unpack + loss-scale update)",
        "value": n_elems / (ms * 1e-3) / 1e9,
        "unit": "Gelem/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "step_ms": r["step_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "scaled_from": scaled_from, "n_elems": n_elems, "n_tensors": len(w.numel),
                   "chunk_elems": w.chunk_elems,
                   "n_chunks": st.nch, "host_resident_chunks": st.n_host, "host_chunks_on_host_cores": st.n_cpu,
                   "loss_scale": w.loss_scale,
                   "weight_decay": w.weight_decay, "fused_check": not a.separate_check, "fused_unpack": a.fused_unpack, "chunk_reuse": a.chunk_reuse,
                   "skipped_steps": r["skipped"]},
        "roofline": roofline,
        "adam_only_gelem_s": adam_elems / (phase["adam_ms"] * 1e-3) / 1e9 if phase["adam_ms"] > 0 else None,
        "phase_ms": phase,
        "cpu_baseline": cpu,
    }
    if on_device:
        out["step_state_on_device"] = on_device
    if st.n_host:
        out["host_link"] = host_link_report(st, r, host_mode)
    if plans:
        out["residency"] = residency_report(r, w, host_fraction)
    if a.sweep_wg:
        out["wg_per_cu_sweep"] = sweep_wg(st, [int(x) for x in a.sweep_wg.split(",")])
    if legs:
        # the other halves of the metric, each a short run of its own after the timed headline:
        # the paper's chunk-reuse layout, host-resident chunks over the link, and on the host cores
        out["fused_unpack"] = leg_fused_unpack(st)
        out["tensors_as_views"] = leg_views(st)
        out["chunk_reuse"] = leg_chunk_reuse(st)
    release(st)
    if a.placements:
        out["placement_trials"] = placement_trials(a, dev, a.placements)
    if legs:
        # each in a process of its own, started after this one has freed its buffers: a workload set up in a
        # fresh process gets its chunk lists placed in HBM as a real run would, and 220 GB of GPT-12.6B fit
        out["launch_bound"] = run_leg("launch_bound")
        out["ragged_packing"] = run_leg("ragged_packing")
        host = run_leg("host")
        out["host_link"], out["host_cores"] = (host.get("host_link"), host.get("host_cores")) if "error" not in host else (host, None)
        out["moving_residency"] = run_leg("moving_residency")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
