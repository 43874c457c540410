"""Pins for the oracle's pack/unpack (byte copies into chunk slots) and the
inf/nan overflow flag."""
import numpy as np

from paper_2108_05818_amd import workloads as W


def _mk_chunks(nch, C, dtype, fill):
    return [np.full(C, fill, dtype=dtype) for _ in range(nch)]


def test_pack_global_index_pattern(orc):
    # pack x[i][k] = running global index: every used chunk prefix becomes a known ramp,
    # with a jump only where a fragment was skipped
    numel = [5, 0, 7, 3, 20, 1, 8, 2]
    C = 8
    slots, used = orc.chunk_layout(numel, C)
    tensors, g = [], 0
    for s in numel:
        tensors.append(np.arange(g, g + s, dtype=np.uint32))
        g += s
    chunks = _mk_chunks(len(used), C, np.uint32, 0xDEADBEEF)
    orc.pack(tensors, slots, chunks, C)
    flat = np.concatenate([c[:int(u)] for c, u in zip(chunks, used)])
    assert np.array_equal(flat, np.arange(g, dtype=np.uint32))          # order kept, nothing lost
    for c, u in zip(chunks, used):
        assert np.all(c[int(u):] == 0xDEADBEEF)                         # fragments untouched
    # each tensor sits where its slot says
    for i, t in enumerate(tensors):
        lin = slots[i].chunk * C + slots[i].offset
        virt = np.concatenate(chunks)
        assert np.array_equal(virt[lin:lin + t.size], t)


def test_pack_unpack_roundtrip_f16_f32(orc):
    rng = np.random.default_rng(5)
    numel = [int(x) for x in rng.integers(0, 300, size=60)] + [1000, 1, 1, 513]
    C = 256
    slots, used = orc.chunk_layout(numel, C)
    for dtype in (np.uint16, np.float32):
        tensors = [rng.integers(0, 60000, size=s).astype(dtype) for s in numel]
        chunks = _mk_chunks(len(used), C, dtype, 77)
        orc.pack(tensors, slots, chunks, C)
        out = [np.zeros(s, dtype) for s in numel]
        orc.unpack(out, slots, chunks, C)
        for a, b in zip(tensors, out):
            assert a.tobytes() == b.tobytes()
        for c, u in zip(chunks, used):
            assert np.all(c[int(u):] == 77)


def test_overflow_flag_vs_numpy_isfinite(orc):
    rng = np.random.default_rng(9)
    for trial in range(50):
        nch = int(rng.integers(1, 6))
        C = 64
        used = rng.integers(0, C + 1, size=nch).astype(np.uint64)
        chunks = [rng.integers(0, 1 << 16, size=C).astype(np.uint16) for _ in range(nch)]
        if trial % 2:          # mostly-finite data with a few planted specials
            chunks = [np.where((c & 0x7C00) == 0x7C00, c & 0x3FFF, c).astype(np.uint16) for c in chunks]
            for _ in range(int(rng.integers(0, 3))):
                k = int(rng.integers(0, nch))
                chunks[k][int(rng.integers(0, C))] = rng.choice(W.specials_f16())
        flag, per = orc.overflow_check(chunks, used)
        want = [int(not np.all(np.isfinite(c[:int(u)].view(np.float16)))) for c, u in zip(chunks, used)]
        assert list(per) == want
        assert flag == int(any(want))


def test_overflow_positions_and_padding(orc):
    C = 32
    used = np.array([32, 17, 1], dtype=np.uint64)
    for special in W.specials_f16():
        for (c, k, expect) in [(0, 0, 1), (0, 31, 1), (1, 16, 1), (2, 0, 1),
                               (1, 17, 0), (1, 31, 0), (2, 1, 0)]:      # last three: padding
            chunks = [np.full(C, 0x3C00, np.uint16) for _ in range(3)]
            chunks[c][k] = special
            flag, per = orc.overflow_check(chunks, used)
            assert flag == expect
            assert per[c] == expect and per.sum() == expect


def test_overflow_max_finite_is_not_flagged(orc):
    chunks = [np.array([0x7BFF, 0xFBFF, 0x0001, 0x8001, 0x0000, 0x8000, 0x03FF], np.uint16)]
    flag, per = orc.overflow_check(chunks, np.array([7], np.uint64))
    assert flag == 0 and per[0] == 0


def test_pack_into_a_sample_of_chunks_equals_full_pack(orc):
    rng = np.random.default_rng(15)
    numel = [int(x) for x in rng.integers(0, 200, size=40)] + [700, 3]
    C = 128
    slots, used = orc.chunk_layout(numel, C)
    tensors = [rng.integers(0, 60000, size=s).astype(np.uint16) for s in numel]
    full = _mk_chunks(len(used), C, np.uint16, 9)
    orc.pack(tensors, slots, full, C)
    keep = set(int(k) for k in rng.choice(len(used), size=len(used) // 2, replace=False))
    part = [np.full(C, 9, np.uint16) if k in keep else None for k in range(len(used))]
    orc.pack(tensors, slots, part, C)
    for k in keep:
        assert part[k].tobytes() == full[k].tobytes()
    out_full = [np.zeros(s, np.uint16) for s in numel]
    out_part = [np.zeros(s, np.uint16) for s in numel]
    orc.unpack(out_full, slots, full, C)
    orc.unpack(out_part, slots, part, C)
    for i, s in enumerate(numel):      # elements living in kept chunks come back, the others stay zero
        lin = slots[i].chunk * C + slots[i].offset + np.arange(s)
        inside = np.isin(lin // C, list(keep))
        assert np.array_equal(out_part[i][inside], out_full[i][inside])
        assert not out_part[i][~inside].any()
