"""The step state on the device (t, loss scale, running beta^t, step-wide scalars) against the oracle's host
bookkeeping, and the whole step recorded into a HIP graph: every replay is one more training step and must
equal the free-running oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2108_05818_amd import psx
from paper_2108_05818_amd import workloads as W

from gpu_util import DEV, ChunkLists, bits16, from_bits16

pytestmark = pytest.mark.gpu

HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, adamw_mode=0)


def scaler_tuple(s):
    return (s.scale, s.good_steps, s.step)


@pytest.mark.parametrize("alias", [False, True])
@pytest.mark.parametrize("clear", [False, True])
def test_device_step_state_follows_the_oracle_scaler(orc, alias, clear):
    """40 steps over a ragged chunk list, overflows planted at chosen steps, growth interval 3: the update takes
    t and the loss scale from the device, the bookkeeping runs on the device, nothing is read back inside a step.
    clear: the flags are cleared by the bookkeeping kernel (PSX_ADVANCE_CLEAR_FLAGS) instead of a reset per step."""
    w = W.config1_tiny()
    slots, used = psx.psx_chunk_layout(w.numel, w.chunk_elems)
    o_slots, _ = orc.chunk_layout(w.numel, w.chunk_elems)
    Cn, nch = w.chunk_elems, len(used)
    ctx = psx.psx_ctx_create(max_chunks=nch, max_tensors=len(w.numel))
    try:
        cl = ChunkLists(used, Cn, alias=alias)
        p_np = [W.params_np(s, 4100 + i) for i, s in enumerate(w.numel)]
        psx.psx_pack(ctx, psx.PSX_F32, [torch.from_numpy(a).to(DEV) for a in p_np], slots, cl.p32, Cn)
        orc.pack(p_np, o_slots, cl.np["p32"], Cn)
        for k in range(nch):
            cl.set("m", k, np.zeros(used[k], np.float32))
            cl.set("v", k, np.zeros(used[k], np.float32))
        o_scaler = orc.scaler(1024.0, 3)
        hyper = psx.make_hyper(**HP)
        psx.psx_step_state_init(ctx, hyper, psx.make_scaler(1024.0, 3))
        chunks = psx.make_chunks(cl.specs())
        rng = np.random.default_rng(41)
        bad_steps = {4, 5, 17, 30}
        for it in range(40):
            g_np = [W.grads_f16_np(s, 4200 + 100 * it + i, o_scaler.scale) for i, s in enumerate(w.numel)]
            if it in bad_steps:
                i = int(rng.integers(0, len(w.numel)))
                g_np[i][int(rng.integers(0, w.numel[i]))] = rng.choice(W.specials_f16())
            if not clear or it == 0:
                psx.psx_overflow_reset(ctx)
            psx.psx_pack(ctx, psx.PSX_F16, [from_bits16(a) for a in g_np], slots, cl.g16, Cn, flags=psx.PSX_PACK_CHECK_OVERFLOW)
            psx.psx_chunk_adam_step(ctx, chunks, hyper, psx.PSX_STEP_USE_FLAG | psx.PSX_STEP_DEVICE_STATE)
            psx.psx_step_state_advance(ctx, psx.PSX_ADVANCE_CLEAR_FLAGS if clear else 0)
            if clear:
                flag_now, per_chunk = psx.psx_overflow_read(ctx, nch)
                assert flag_now == 0 and not any(per_chunk)
            # the oracle, free-running, with its host scaler
            orc.pack(g_np, o_slots, cl.np["g16"], Cn)
            o_flag = cl.oracle_step(orc, orc.hyper(step=o_scaler.step, loss_scale=o_scaler.scale, **HP))
            orc.scaler_update(o_scaler, o_flag)
            assert o_flag == int(it in bad_steps)
            if it % 5 == 4 or it in bad_steps or it == 39:
                s, last_flag, skipped = psx.psx_step_state_read(ctx)
                assert scaler_tuple(s) == scaler_tuple(o_scaler) and last_flag == o_flag
                assert skipped == sum(1 for b in bad_steps if b <= it)
                assert cl.compare(f"step {it}") == 0.0
        assert o_scaler.scale != 1024.0 and o_scaler.step == 41 - len(bad_steps)
        # the host-scalar path and the device-state path agree on what the next update is
        with pytest.raises(psx.PsxError):                              # other hyper-parameters than the state was set up with
            psx.psx_chunk_adam_step(ctx, chunks, psx.make_hyper(**dict(HP, lr=2e-3)), psx.PSX_STEP_DEVICE_STATE)
    finally:
        psx.psx_ctx_destroy(ctx)


def test_device_scalars_equal_the_oracles_over_twenty_thousand_steps(orc):
    """beta^t as a running product and the double-precision division and square root on the device must give
    the oracle's fp32 scalars at every step: one wrong bit in any of them would leave p, m or v different
    from the oracle's for good.  20 000 updates of a 96-element chunk, compared in full at checkpoints."""
    n = 96
    ctx = psx.psx_ctx_create(max_chunks=1, max_tensors=1)
    try:
        cl = ChunkLists([n], 128)
        cl.set("p32", 0, W.params_np(n, 51))
        cl.set("m", 0, np.zeros(n, np.float32))
        cl.set("v", 0, np.zeros(n, np.float32))
        cl.set("g16", 0, W.grads_f16_np(n, 52, 64.0))
        hyper = psx.make_hyper(**HP)
        psx.psx_step_state_init(ctx, hyper, psx.make_scaler(64.0, 1 << 30))
        chunks = psx.make_chunks(cl.specs())
        psx.psx_overflow_reset(ctx)
        checkpoints = {1, 2, 3, 10, 100, 1000, 5000, 12345, 20000}
        for t in range(1, 20001):
            psx.psx_chunk_adam_step(ctx, chunks, hyper, psx.PSX_STEP_USE_FLAG | psx.PSX_STEP_DEVICE_STATE)
            psx.psx_step_state_advance(ctx)
            cl.oracle_step(orc, orc.hyper(step=t, loss_scale=64.0, **HP))
            if t in checkpoints:
                torch.cuda.synchronize()
                assert cl.compare(f"t={t}") == 0.0
        s, _, skipped = psx.psx_step_state_read(ctx)
        assert (s.scale, s.step, skipped) == (64.0, 20001, 0)
    finally:
        psx.psx_ctx_destroy(ctx)


def test_state_initialised_in_the_middle_of_a_run(orc):
    """A state set up at t = 777 with 2 good steps behind it continues exactly where a host scaler would."""
    n = 300
    ctx = psx.psx_ctx_create(max_chunks=1, max_tensors=1)
    try:
        cl = ChunkLists([n], 512)
        cl.set("p32", 0, W.params_np(n, 61))
        cl.set("m", 0, W.params_np(n, 62) * np.float32(0.05))
        cl.set("v", 0, np.abs(W.params_np(n, 63)) * np.float32(1e-4))
        sc = psx.make_scaler(256.0, 4)
        sc.step, sc.good_steps = 777, 2
        o_scaler = orc.scaler(256.0, 4)
        o_scaler.step, o_scaler.good_steps = 777, 2
        hp = dict(HP, adamw_mode=1, weight_decay=0.1)
        hyper = psx.make_hyper(**hp)
        psx.psx_step_state_init(ctx, hyper, sc)
        chunks = psx.make_chunks(cl.specs())
        for it in range(6):
            cl.set("g16", 0, W.grads_f16_np(n, 64 + it, o_scaler.scale))
            psx.psx_chunk_adam_step(ctx, chunks, hyper, psx.PSX_STEP_CHECK_FIRST | psx.PSX_STEP_DEVICE_STATE)
            psx.psx_step_state_advance(ctx)
            o_flag = cl.oracle_step(orc, orc.hyper(step=o_scaler.step, loss_scale=o_scaler.scale, **hp))
            orc.scaler_update(o_scaler, o_flag)
            s, _, _ = psx.psx_step_state_read(ctx)
            assert scaler_tuple(s) == scaler_tuple(o_scaler)
            assert cl.compare(f"it {it}") == 0.0
        assert o_scaler.scale == 1024.0
    finally:
        psx.psx_ctx_destroy(ctx)


def test_whole_step_recorded_into_a_graph_and_replayed(orc):
    """Overflow reset, gradient pack with the overflow test, update from the device state, fp16 unpack and the
    bookkeeping are recorded once into a HIP graph; each replay is a training step of its own (new gradients
    are written into the same gradient tensors between replays, one of them with an inf), with eager work and
    synchronisations in between, and every replay is compared with the free-running oracle."""
    w = W.config1_tiny()
    slots, used = psx.psx_chunk_layout(w.numel, w.chunk_elems)
    o_slots, _ = orc.chunk_layout(w.numel, w.chunk_elems)
    Cn, nch = w.chunk_elems, len(used)
    ctx = psx.psx_ctx_create(max_chunks=nch, max_tensors=len(w.numel))
    try:
        cl = ChunkLists(used, Cn)
        p_np = [W.params_np(s, 7100 + i) for i, s in enumerate(w.numel)]
        psx.psx_pack(ctx, psx.PSX_F32, [torch.from_numpy(a).to(DEV) for a in p_np], slots, cl.p32, Cn)
        orc.pack(p_np, o_slots, cl.np["p32"], Cn)
        for k in range(nch):
            cl.set("m", k, np.zeros(used[k], np.float32))
            cl.set("v", k, np.zeros(used[k], np.float32))
        o_scaler = orc.scaler(1024.0, 2)
        hyper = psx.make_hyper(**HP)
        psx.psx_step_state_init(ctx, hyper, psx.make_scaler(1024.0, 2))
        chunks = psx.make_chunks(cl.specs())
        g_t = [torch.zeros(s, dtype=torch.float16, device=DEV) for s in w.numel]      # the gradient tensors a backward pass would fill
        out_t = [torch.zeros(s, dtype=torch.float16, device=DEV) for s in w.numel]
        g_ptrs, o_ptrs, c16 = psx.ptr_array(g_t), psx.ptr_array(out_t), psx.ptr_array(cl.g16)
        p16_ptrs = psx.ptr_array(cl.p16)

        def one_step():
            psx.psx_overflow_reset(ctx)
            psx.psx_pack(ctx, psx.PSX_F16, g_ptrs, slots, cl.g16, Cn, flags=psx.PSX_PACK_CHECK_OVERFLOW, n=len(g_t))
            psx.psx_chunk_adam_step(ctx, chunks, hyper, psx.PSX_STEP_USE_FLAG | psx.PSX_STEP_DEVICE_STATE)
            psx.psx_unpack(ctx, psx.PSX_F16, o_ptrs, slots, cl.p16, Cn, n=len(out_t))
            psx.psx_step_state_advance(ctx)

        def new_gradients(it, plant=False):
            g_np = [W.grads_f16_np(s, 7200 + 100 * it + i, o_scaler.scale) for i, s in enumerate(w.numel)]
            if plant:
                g_np[5][3] = 0x7C00
            for t, a in zip(g_t, g_np):
                t.copy_(from_bits16(a))
            return g_np

        def oracle_follows(g_np, tag):
            orc.pack(g_np, o_slots, cl.np["g16"], Cn)
            o_flag = cl.oracle_step(orc, orc.hyper(step=o_scaler.step, loss_scale=o_scaler.scale, **HP))
            orc.scaler_update(o_scaler, o_flag)
            torch.cuda.synchronize()
            assert cl.compare(tag) == 0.0
            o_out = [np.zeros(s, np.uint16) for s in w.numel]
            orc.unpack(o_out, o_slots, cl.np["p16"], Cn)
            for a, b in zip(out_t, o_out):
                assert bits16(a).tobytes() == b.tobytes(), tag
            s, last_flag, _ = psx.psx_step_state_read(ctx)
            assert scaler_tuple(s) == scaler_tuple(o_scaler) and last_flag == o_flag
            return o_flag

        # one eager step first: it uploads the descriptor tables the recorded calls will find unchanged
        oracle_follows((new_gradients(0), one_step())[0], "eager step")
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_step()
            # what cannot be recorded is refused and leaves the capture intact
            with pytest.raises(psx.PsxError) as e:
                psx.psx_chunk_adam_step(ctx, chunks, hyper, psx.PSX_STEP_USE_FLAG)           # host t and scale would be frozen
            assert e.value.code == psx.PSX_ECAPTURE
            with pytest.raises(psx.PsxError) as e:
                psx.psx_overflow_read(ctx)
            assert e.value.code == psx.PSX_ECAPTURE
            with pytest.raises(psx.PsxError) as e:                                           # another tensor list: a table upload
                psx.psx_pack(ctx, psx.PSX_F16, g_t[:3], slots, cl.g16, Cn)
            assert e.value.code == psx.PSX_ECAPTURE
        # capture runs nothing: the state is where the eager step left it
        s, _, _ = psx.psx_step_state_read(ctx)
        assert scaler_tuple(s) == scaler_tuple(o_scaler)
        flags = []
        for it in range(1, 9):
            g_np = new_gradients(it, plant=it in (3, 6))
            junk = torch.randn(1 << 16, device=DEV).sum()                  # unrelated eager work between replays
            graph.replay()
            flags.append(oracle_follows(g_np, f"replay {it}"))
            assert torch.isfinite(junk)
        assert flags == [0, 0, 1, 0, 0, 1, 0, 0] and o_scaler.scale != 1024.0
        # and an eager step after the replays continues from the same state
        oracle_follows((new_gradients(9), one_step())[0], "eager step after the replays")
    finally:
        psx.psx_ctx_destroy(ctx)
