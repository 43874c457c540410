"""Helpers for the GPU parity tests: chunk lists on the device with numpy
mirrors for the oracle.  Both sides are filled from the same seeded arrays; the
oracle then runs free on its mirror (it never sees anything the HIP path
produced) and the two are compared after every step."""
import numpy as np
import torch

SENT32 = 0x7FC12345   # a NaN payload: padding must keep it
SENT16 = 0x7E55

DEV = "cuda"


def bits16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def bits32(t):
    return t.view(torch.int32).cpu().numpy().view(np.uint32)


def f32(t):
    return t.cpu().numpy()


def from_bits16(a, device=DEV):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.float16)


def sent32(n):
    return np.full(n, SENT32, np.uint32).view(np.float32)


def sent16(n):
    return np.full(n, SENT16, np.uint16)


def ulp32(x):
    x = np.abs(np.asarray(x, dtype=np.float32))
    x = np.maximum(x, np.float32(1.1754944e-38))
    return (np.nextafter(x, np.float32(np.inf)) - x).astype(np.float64)


def err_in_ulps(name, got, want, ref=None, max_ulp=2):
    """0.0 when bit-identical; otherwise the largest |delta| in ulps of the reference magnitude
    (the oracle value, or for params max(|p_old|, |p_new|): under cancellation the error floor is
    an ulp of the operands).  Asserts the 2-ulp bar."""
    got = np.asarray(got); want = np.asarray(want)
    if got.tobytes() == want.tobytes():
        return 0.0
    assert not (np.isnan(got) != np.isnan(want)).any(), f"{name}: NaN pattern differs"
    mag = np.abs(want) if ref is None else np.maximum(np.abs(want), np.abs(ref))
    d = np.abs(got.astype(np.float64) - want.astype(np.float64))
    worst = float(np.nanmax(d / ulp32(mag)))
    assert worst <= max_ulp, f"{name}: {worst} ulp"
    return worst


class ChunkLists:
    """The chunk lists on the device and their numpy mirrors (fp16 as uint16 bit patterns)."""

    NAMES = ("p32", "m", "v", "p16", "g16")

    def __init__(self, used, C, alias=False, device=DEV):
        self.used = [int(u) for u in used]
        self.C = C
        self.n = len(used)
        self.alias = alias
        self.np = dict(p32=[sent32(C) for _ in range(self.n)], m=[sent32(C) for _ in range(self.n)],
                       v=[sent32(C) for _ in range(self.n)], p16=[sent16(C) for _ in range(self.n)])
        self.np["g16"] = self.np["p16"] if alias else [sent16(C) for _ in range(self.n)]
        up32 = lambda a: torch.from_numpy(a.copy()).to(device)
        self.p32 = [up32(a) for a in self.np["p32"]]
        self.m = [up32(a) for a in self.np["m"]]
        self.v = [up32(a) for a in self.np["v"]]
        self.p16 = [from_bits16(a, device) for a in self.np["p16"]]
        self.g16 = self.p16 if alias else [from_bits16(a, device) for a in self.np["g16"]]

    def set(self, name, k, arr, at=0):
        """Write the same seeded values into the mirror and the device chunk."""
        arr = np.ascontiguousarray(arr)
        n = arr.size
        self.np[name][k][at:at + n] = arr
        dev = getattr(self, name)[k]
        if name in ("p16", "g16"):
            dev[at:at + n] = from_bits16(arr.astype(np.uint16), dev.device)
        else:
            dev[at:at + n] = torch.from_numpy(arr.astype(np.float32)).to(dev.device)

    def specs(self, loc=None, host=None):
        out = []
        for k in range(self.n):
            s = dict(g16=self.g16[k], p16=self.p16[k], p32=self.p32[k], m=self.m[k], v=self.v[k], used=self.used[k])
            if loc is not None:
                s["loc_in"], s["loc_out"] = loc[k]
            if host is not None and host[k] is not None:
                s["p32_host"], s["m_host"], s["v_host"] = host[k]
            out.append(s)
        return out

    def oracle_step(self, orc, h):
        """The oracle's whole step on the mirror; returns its flag.  Keeps the old params as
        the reference magnitude of the comparison."""
        self.p_old = [x.copy() for x in self.np["p32"]]
        return orc.chunk_adam_step(self.np["g16"], self.np["p16"], self.np["p32"], self.np["m"], self.np["v"],
                                   np.array(self.used, np.uint64), h)

    def compare(self, tag="", where=None):
        """Device (or `where[k]` = (p32, m, v) buffers, e.g. pinned host) against the mirror, padding
        included.  fp32 states: 2-ulp bar, 0 expected.  p16: bit-exact wherever the fp32 params agree
        bit for bit (it is the fp16 of the GPU's own params).  Returns the worst error in ulps."""
        worst = 0.0
        for k in range(self.n):
            u = self.used[k]
            bufs = (self.p32[k], self.m[k], self.v[k]) if where is None or where[k] is None else where[k]
            got_p = None
            for name, buf in zip(("p32", "m", "v"), bufs):
                got = buf.cpu().numpy()
                want = self.np[name][k]
                assert got[u:].tobytes() == want[u:].tobytes(), f"{tag} chunk {k} {name}: padding touched"
                ref = self.p_old[k][:u] if name == "p32" and hasattr(self, "p_old") else None
                worst = max(worst, err_in_ulps(f"{tag} chunk {k} {name}", got[:u], want[:u], ref))
                if name == "p32":
                    got_p = got
            got16 = bits16(self.p16[k])
            want16 = self.np["p16"][k]
            assert got16[u:].tobytes() == want16[u:].tobytes(), f"{tag} chunk {k} p16: padding touched"
            same = got_p[:u].view(np.uint32) == self.np["p32"][k][:u].view(np.uint32)
            assert np.array_equal(got16[:u][same], want16[:u][same]), f"{tag} chunk {k} p16"
        return worst
