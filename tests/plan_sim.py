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
    items = plan[h["off_items"]:h["off_items"] + 20 * h["n_tiles"] * h["n_items"]].view(np.int32)
    items = items.reshape(h["n_tiles"], h["n_items"], 5)
    dst = plan[h["off_dst_lut"]:h["off_dst_lut"] + 4 * h["n_tiles"] * P4].view(np.int32).reshape(h["n_tiles"], P4)
    bins = h["n_mgroups"] * WM
    perm = plan[h["off_perm"]:h["off_perm"] + 4 * bins * K].view(np.int32).reshape(bins, K)
    seg = plan[h["off_seg"]:h["off_seg"] + 4 * bins * h["n_chunks"] * (1 + K)].view(np.uint32)
    seg = seg.reshape(bins, h["n_chunks"], 1 + K)
    blk = plan[h["off_blk"]:h["off_blk"] + 8 * h["n_mgroups"] * h["n_chunks"]].view(np.uint32)
    blk = blk.reshape(h["n_mgroups"], h["n_chunks"], 2)
    rec = plan[h["off_rec"]:h["off_rec"] + 8 * h["n_records"]]
    rec_off = rec.view(np.uint32)[0::2]
    rec_val = rec.view(np.float32)[1::2]
    assert sorted(perm[perm >= 0].tolist()) == list(range(M)), "perm must cover every row once"
    out = np.full((N, M, h["E"] * h["F"]), np.nan)
    xf = x.reshape(N, C, H * W).astype(np.float64)
    buf_floats = h["buf_floats"]
    assert buf_floats == nslots * CC * NB * ps
    lds_len = buf_floats + h["tail_floats"]            # one window buffer plus the zeroed tail
    assert h["lds_bytes"] == (2 * buf_floats + h["tail_floats"]) * 4 + 2 * h["rec_buf_bytes"]
    threads = 64 * h["WQ"] * WM
    assert h["n_items"] * CC * NB <= 8 * threads
    pos = np.arange(P4)
    for t in range(h["n_tiles"]):
        for n0 in range(0, N, NB):
            nb = min(NB, N - n0)
            acc = np.zeros((bins, K, NB, P4))
            for ch in range(h["n_chunks"]):
                c0 = ch * CC
                ccur = min(CC, C - c0)
                # the frame was zeroed once; the staging items rewrite the words that hold input
                lds = np.zeros(lds_len)
                it = items[t]
                for sidx in range(h["n_items"]):
                    s_src = it[sidx, 0]
                    if s_src < 0:
                        continue
                    for u in range(4):
                        d0 = it[sidx, 1 + u]
                        if d0 < 0:
                            continue
                        for cl in range(ccur):
                            for nl in range(nb):
                                lds[d0 + (cl * NB + nl) * ps] = xf[n0 + nl, c0 + cl, s_src]
                for b in range(bins):
                    mgi = b // WM
                    assert seg[b, ch, 0] + seg[b, ch, 1:].sum() <= blk[mgi, ch, 1]
                    assert (int(blk[mgi, ch, 1]) + 1) * B * 8 <= h["rec_buf_bytes"]
                    at = (int(blk[mgi, ch, 0]) + int(seg[b, ch, 0])) * B
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
