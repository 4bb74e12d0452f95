"""Shared test plumbing: runs the HIP path through the C-ABI binding and the oracle beside it."""
from __future__ import annotations

import numpy as np

TOL = 1e-4  # |gpu - oracle| <= TOL * sum|w*x| per output element (fp32 summation order is free)


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class DeviceLayer:
    """CSR stretched by escoin_sconv_pack and uploaded; input uploaded; buffers allocated."""

    def __init__(self, esc, L, tuning=None):
        import torch
        self.esc, self.L = esc, L
        self.tuning = tuning
        self.desc = esc.desc_of(L.spec)
        self.stretched = esc.escoin_sconv_pack(self.desc, L.rowptr, L.colidx)
        self.d_rowptr = to_dev(L.rowptr)
        self.d_colidx = to_dev(self.stretched) if L.nnz else torch.empty(1, dtype=torch.int32, device="cuda")
        self.d_value = to_dev(L.value) if L.nnz else torch.empty(1, dtype=torch.float32, device="cuda")
        self.d_in = to_dev(L.input)
        self.d_bias = to_dev(L.bias)
        s = L.spec
        self.d_padded = torch.empty(esc.escoin_padded_elems(self.desc), dtype=torch.float32, device="cuda")
        self.d_out = torch.empty((s.N, s.M, s.E, s.F), dtype=torch.float32, device="cuda")

    def pad(self):
        self.d_padded.fill_(float("nan"))
        self.esc.escoin_pad_in(self.desc, self.d_in, self.d_padded)
        return self.d_padded

    def forward_tiled(self, flags=0):
        """The LDS-tiled entry point: plan from the stretched CSR, unpadded input."""
        import torch
        esc = self.esc
        if not hasattr(self, "plan"):
            t = esc.make_tuning(**self.tuning) if self.tuning else None
            self.plan = esc.escoin_sconv_plan_build(self.desc, self.L.rowptr, self.stretched,
                                                    self.L.value, t)
            self.d_plan = to_dev(self.plan)
        self.d_out.fill_(float("nan"))
        esc.escoin_sconv_forward_tiled(self.desc, self.plan, self.d_plan, self.d_in, self.d_out,
                                       self.d_bias, flags)
        torch.cuda.synchronize()
        return self.d_out.cpu().numpy()

    def run(self, path, flags=0):
        return self.forward_tiled(flags) if path == "tiled" else self.forward(flags)

    def forward(self, flags=0):
        import torch
        self.pad()
        self.d_out.fill_(float("nan"))
        self.esc.escoin_sconv_forward(self.desc, self.d_rowptr, self.d_colidx, self.d_value,
                                      self.d_padded, self.d_out, self.d_bias, flags)
        torch.cuda.synchronize()
        return self.d_out.cpu().numpy()


def oracle_full(oracle, L, flags=0):
    s = L.spec
    Wd = oracle.csr_to_dense(s.M, s.C, s.R, s.S, L.rowptr, L.colidx, L.value)
    return oracle.conv(L.input, Wd, s.stride, s.pad, bias=L.bias, flags=flags)


def assert_within_bound(got, ref, bound, what=""):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output (unwritten element?)"
    err = np.abs(got - ref.astype(np.float64))
    lim = TOL * bound
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements outside 1e-4*sum|w*x|; "
                             f"worst at {i}: got {got[i]!r} ref {ref[i]!r} bound {bound[i]!r}")
    return float((err / np.maximum(bound, 1e-30)).max())


def sample_points(spec, k, seed):
    """k random (n, m, h, w) plus the corners/edges of the first and last image/channel."""
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(0, spec.N, k), rng.integers(0, spec.M, k),
                    rng.integers(0, spec.E, k), rng.integers(0, spec.F, k)], axis=1)
    edge = [(n, m, h, w) for n in (0, spec.N - 1) for m in (0, spec.M - 1)
            for h in (0, spec.E - 1) for w in (0, spec.F - 1)]
    return np.concatenate([pts, np.array(edge)], axis=0).astype(np.int32)


def seam_points(spec, plan_info, seed, pairs=24):
    """Output elements on both sides of every seam of the tiling: the last row of a band and the
    first row of the next (all columns), and, where several images share a tile, the images on
    both sides of a tile boundary and the last image (whole maps), for `pairs` random (image,
    channel) pairs each."""
    rng = np.random.default_rng(seed)
    TH, NB = plan_info["TH"], plan_info["NB"]
    pts = []
    rows = sorted({h for k in range(1, -(-spec.E // TH)) for h in (k * TH - 1, k * TH) if 0 <= h < spec.E})
    for _ in range(pairs):
        n, m = int(rng.integers(0, spec.N)), int(rng.integers(0, spec.M))
        pts += [(n, m, h, w) for h in rows for w in range(spec.F)]
    if NB > 1:
        images = sorted({n for n in (NB - 1, NB, (spec.N // NB) * NB - 1, (spec.N // NB) * NB, spec.N - 1)
                         if 0 <= n < spec.N})
        for n in images:
            for m in rng.integers(0, spec.M, size=max(1, pairs // 4)):
                pts += [(n, int(m), h, w) for h in range(spec.E) for w in range(spec.F)]
    return np.array(pts, dtype=np.int32).reshape(-1, 4)


def random_layers_and_tunings(wl, seed, count):
    """Seeded random small layers (any filter size, stride, padding) with random tiling knobs."""
    rng = np.random.default_rng(seed)
    for it in range(count):
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        stride, pad = int(rng.choice([1, 1, 1, 2, 3])), int(rng.integers(0, 4))
        H = int(rng.integers(max(1, R - 2 * pad), 20))
        W = int(rng.integers(max(1, S - 2 * pad), 30))
        N, C, M = int(rng.integers(1, 9)), int(rng.integers(1, 7)), int(rng.integers(1, 10))
        L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, float(rng.choice([0.0, 0.5, 0.9])),
                            seed=5000 + it, dist="normal")
        tune = {}
        if rng.random() < 0.7:
            tune["K"], tune["Q"] = [(1, 1), (1, 2), (2, 1), (2, 2), (4, 1), (4, 2), (8, 1)][int(rng.integers(0, 7))]
        if rng.random() < 0.5:
            tune["WM"] = int(rng.integers(1, 5))
        if rng.random() < 0.5:
            tune["CC"] = int(rng.integers(1, C + 1))
        if rng.random() < 0.4:
            tune["NB"] = int(rng.integers(1, N + 1))
        elif rng.random() < 0.4:
            tune["TH"] = int(rng.integers(1, L.spec.E + 1))
        if rng.random() < 0.3:
            tune["CS"] = int(rng.integers(1, 4))
        if rng.random() < 0.4:
            tune["WS"] = int(rng.integers(1, 5))
        if rng.random() < 0.3:
            tune["CC0"] = int(rng.integers(1, C + 1))
        yield L, tune
