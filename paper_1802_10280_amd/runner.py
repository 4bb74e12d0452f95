"""Per-layer driver used by the bench, the smoke check and the tests: packs the CSR once,
uploads it, owns the torch device buffers and issues the library calls of one forward pass.
It only marshals arguments; every step of the path runs inside libescoin.so."""
from __future__ import annotations

import numpy as np

from . import binding as B


class LayerRunner:
    def __init__(self, layer, path: str = "auto", flags: int = 0, stream=None, tuning=None, d_in=None):
        """d_in: a device tensor to read the input from instead of uploading the layer's own
        (the previous layer's output when layers are chained)."""
        import torch
        self.layer, self.flags, self.stream = layer, flags, stream
        s = layer.spec
        self.desc = B.desc_of(s)
        self.stretched = B.escoin_sconv_pack(self.desc, layer.rowptr, layer.colidx)
        dev = "cuda"
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        nz = layer.nnz > 0
        self.d_rowptr = up(layer.rowptr)
        self.d_colidx = up(self.stretched) if nz else torch.zeros(1, dtype=torch.int32, device=dev)
        self.d_value = up(layer.value) if nz else torch.zeros(1, dtype=torch.float32, device=dev)
        self.d_bias = up(layer.bias) if layer.bias is not None else None
        if d_in is not None:
            assert tuple(d_in.shape) == (s.N, s.C, s.H, s.W) and d_in.dtype == torch.float32
            self.d_in = d_in
        else:
            self.d_in = up(layer.input)
        self.d_padded = torch.empty(B.escoin_padded_elems(self.desc), dtype=torch.float32, device=dev)
        self.d_out = torch.empty((s.N, s.M, s.E, s.F), dtype=torch.float32, device=dev)
        self.path = "tiled" if path == "auto" else path
        if self.path == "tiled":
            if isinstance(tuning, dict):
                tuning = B.make_tuning(**tuning)
            self.plan = B.escoin_sconv_plan_build(self.desc, layer.rowptr, self.stretched,
                                                  layer.value, tuning)
            self.plan_info = B.plan_header(self.plan)
            self.d_plan = up(self.plan)
        elif self.path != "direct":
            raise ValueError(f"unknown sconv path {path!r}")

    @staticmethod
    def available_paths(layer):
        return ["tiled", "direct"]

    # -- one forward pass ---------------------------------------------------------------
    def pad_in(self):
        B.escoin_pad_in(self.desc, self.d_in, self.d_padded, self.stream)

    def sconv(self):
        B.escoin_sconv_forward(self.desc, self.d_rowptr, self.d_colidx, self.d_value,
                               self.d_padded, self.d_out, self.d_bias, self.flags, self.stream)

    def sconv_tiled(self):
        B.escoin_sconv_forward_tiled(self.desc, self.plan, self.d_plan, self.d_in, self.d_out,
                                     self.d_bias, self.flags, self.stream)

    def kernels(self):
        """The library calls of one forward pass, in order (the tiled path pads while staging,
        so it has no separate pad_in)."""
        return [self.sconv_tiled] if self.path == "tiled" else [self.pad_in, self.sconv]

    def kernel_names(self):
        return ["sconv"] if self.path == "tiled" else ["pad_in", "sconv"]

    def sconv_kernel_name(self):
        if self.path == "tiled":
            h = self.plan_info
            vw = h["VW"] if self.d_in.data_ptr() % 16 == 0 else 1
            if vw == 4 and h["n_dma"] > 0 and h["WW"] == 4:
                vw = 16       # staged by global -> LDS copies
            return f"sconv_tiled_kernel<{h['K']}, {h['Q']}, {h['B']}, {vw}>"
        return "sconv_direct_kernel"

    def run(self):
        for k in self.kernels():
            k()
        return self.d_out
