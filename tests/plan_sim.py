"""Host-side emulation of the tiled kernel's data flow from a plan blob (numpy, fp64).

Walks the plan exactly as the kernel does -- stage the LDS window through src_lut, gather-MAC
the records of every (row bin, chunk), scatter through dst_lut and the row permutation -- so a
wrong table, offset or segment in the plan shows up on the CPU, before any GPU run."""
import numpy as np

import paper_1802_10280_amd as esc


def simulate(plan: np.ndarray, x: np.ndarray, M: int) -> np.ndarray:
    h = esc.plan_header(plan)
    N, C, H, W = x.shape
    assert (C, H, W, M) == (h["C"], h["H"], h["W"], h["M"])
    K, B, WM, CC, NB = h["K"], h["B"], h["WM"], h["CC"], h["NB"]
    ps, P4, nslots = h["plane_stride"], h["P4"], h["n_slots"]
    src = plan[h["off_src_lut"]:h["off_src_lut"] + 4 * h["n_tiles"] * h["lut_entries"]].view(np.int32)
    src = src.reshape(h["n_tiles"], nslots, ps)
    dst = plan[h["off_dst_lut"]:h["off_dst_lut"] + 4 * h["n_tiles"] * P4].view(np.int32).reshape(h["n_tiles"], P4)
    bins = h["n_mgroups"] * WM
    perm = plan[h["off_perm"]:h["off_perm"] + 4 * bins * K].view(np.int32).reshape(bins, K)
    seg = plan[h["off_seg"]:h["off_seg"] + 4 * bins * h["n_chunks"] * (1 + K)].view(np.uint32)
    seg = seg.reshape(bins, h["n_chunks"], 1 + K)
    rec = plan[h["off_rec"]:h["off_rec"] + 8 * h["n_records"]]
    rec_off = rec.view(np.uint32)[0::2]
    rec_val = rec.view(np.float32)[1::2]
    assert sorted(perm[perm >= 0].tolist()) == list(range(M)), "perm must cover every row once"
    out = np.full((N, M, h["E"] * h["F"]), np.nan)
    xf = x.reshape(N, C, H * W).astype(np.float64)
    lds_len = h["lds_floats"]
    pos = np.arange(P4)
    for t in range(h["n_tiles"]):
        for n0 in range(0, N, NB):
            nb = min(NB, N - n0)
            acc = np.zeros((bins, K, NB, P4))
            for ch in range(h["n_chunks"]):
                c0 = ch * CC
                ccur = min(CC, C - c0)
                lds = np.full(lds_len, np.nan)      # unstaged LDS is garbage
                win = np.zeros((nslots, CC, NB, ps))
                win[:, ccur:] = np.nan
                win[:, :, nb:] = 0.0
                for sl in range(nslots):
                    s = src[t, sl]
                    ok = s >= 0
                    v = np.where(ok[None, None, :], xf[n0:n0 + nb, c0:c0 + ccur][:, :, np.where(ok, s, 0)], 0.0)
                    win[sl, :ccur, :nb] = v.transpose(1, 0, 2)
                lds[:win.size] = win.ravel()
                for b in range(bins):
                    at = int(seg[b, ch, 0]) * B
                    for k in range(K):
                        cnt = int(seg[b, ch, 1 + k]) * B
                        for j in range(at, at + cnt):
                            off = int(rec_off[j])
                            assert off % 16 == 0
                            o = off // 4
                            for nl in range(NB):
                                idx = o + nl * ps + pos
                                assert idx.max() + 3 < lds_len
                                acc[b, k, nl] += float(rec_val[j]) * lds[idx]
                        at += cnt
            d = dst[t]
            ok = d >= 0
            for b in range(bins):
                for k in range(K):
                    m = perm[b, k]
                    if m < 0:
                        continue
                    for nl in range(nb):
                        assert np.isnan(out[n0 + nl, m, d[ok]]).all(), "output written twice"
                        out[n0 + nl, m, d[ok]] = acc[b, k, nl, ok]
    assert not np.isnan(out).any(), "some output element was never written or read garbage"
    return out.reshape(N, M, h["E"], h["F"])
