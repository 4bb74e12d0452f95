"""Host-side emulation of the tiled kernel's data flow from a plan blob (numpy, fp64).

Walks the plan exactly as the kernel does -- stage the LDS window through the item table,
walk the records of every (row bin, chunk, row, alignment class) with the lane table and the
neighbour-lane shifts, scatter through dst_lut and the row permutation -- so a wrong table,
offset, class or segment in the plan shows up on the CPU, before any GPU run."""
import numpy as np

import paper_1802_10280_amd as esc

NCLS = 4


def _window_words(x, cls):
    """x: (64, 4) groups fetched by the 64 lanes of a run; returns the (64, 4) words each lane
    multiplies.  Lanes past either end receive 0 from the lane shift."""
    nxt = np.vstack([x[1:], np.zeros((1, 4))])       # value held by lane + 1
    prv = np.vstack([np.zeros((1, 4)), x[:-1]])      # value held by lane - 1
    if cls == 0:
        return x
    if cls == 1:
        return np.stack([x[:, 1], x[:, 2], x[:, 3], nxt[:, 0]], axis=1)
    if cls == 2:
        return np.stack([x[:, 2], x[:, 3], nxt[:, 0], nxt[:, 1]], axis=1)
    return np.stack([prv[:, 3], x[:, 0], x[:, 1], x[:, 2]], axis=1)


def simulate(plan: np.ndarray, x: np.ndarray, M: int) -> np.ndarray:
    h = esc.plan_header(plan)
    N, C, H, W = x.shape
    assert (C, H, W, M) == (h["C"], h["H"], h["W"], h["M"])
    K, Q, B, WM, WQ, CC, NB = h["K"], h["Q"], h["B"], h["WM"], h["WQ"], h["CC"], h["NB"]
    ps, P4 = h["plane_stride"], h["P4"]
    threads = 64 * WQ * WM
    # staging slots: [tile][slot][thread] of (src offset, LDS byte | channel << 18)
    slots = plan[h["off_items"]:h["off_items"] + 8 * h["n_tiles"] * 12 * threads].view(np.uint32)
    slots = slots.reshape(h["n_tiles"], 12 * threads, 2)
    runs = WQ * Q
    lanes = plan[h["off_lanes"]:h["off_lanes"] + 12 * runs * 64].view(np.int32).reshape(runs, 64, 3)
    dst = plan[h["off_dst_lut"]:h["off_dst_lut"] + 4 * h["n_tiles"] * P4].view(np.int32).reshape(h["n_tiles"], P4)
    bins = h["n_mgroups"] * WM
    # accumulator rows: (output channel, region it lends a partial sum to, first region and
    # count of the partial sums it collects), then the number of regions of every channel group
    rows = plan[h["off_perm"]:h["off_perm"] + 16 * bins * K].view(np.int32).reshape(bins, K, 4)
    group_regions = plan[h["off_perm"] + 16 * bins * K:h["off_perm"] + 16 * bins * K + 4 * h["n_mgroups"]].view(np.int32)
    perm = rows[:, :, 0]
    CC0, ZF = h["CC0"], h["zero_floats"]
    assert 1 <= CC0 <= CC and h["n_chunks"] == (1 if C <= CC0 else 1 + -(-(C - CC0) // CC))
    assert 1 <= h["WS"] <= WM
    sw = 1 + K * NCLS
    seg = plan[h["off_seg"]:h["off_seg"] + 4 * bins * h["n_chunks"] * sw].view(np.uint32)
    seg = seg.reshape(bins, h["n_chunks"], sw)
    blk = plan[h["off_blk"]:h["off_blk"] + 8 * h["n_mgroups"] * h["n_chunks"]].view(np.uint32)
    blk = blk.reshape(h["n_mgroups"], h["n_chunks"], 2)
    rec = plan[h["off_rec"]:h["off_rec"] + 8 * h["n_records"]]
    rec_off = rec.view(np.uint32)[0::2]
    rec_val = rec.view(np.float32)[1::2]
    owners = rows[(rows[:, :, 0] >= 0) & (rows[:, :, 1] < 0)]
    assert sorted(owners[:, 0].tolist()) == list(range(M)), "every output channel needs exactly one owning row"
    for mgi in range(h["n_mgroups"]):
        grp = rows[mgi * WM:(mgi + 1) * WM].reshape(-1, 4)
        lend = grp[(grp[:, 0] >= 0) & (grp[:, 1] >= 0)]
        assert sorted(lend[:, 1].tolist()) == list(range(group_regions[mgi])), "regions of a group: one lender each"
        assert group_regions[mgi] <= h["max_regions"]
        for m_, _, first, cnt in grp[(grp[:, 0] >= 0) & (grp[:, 1] < 0)]:
            assert (lend[(lend[:, 1] >= first) & (lend[:, 1] < first + cnt), 0] == m_).all() and \
                   (lend[:, 0] == m_).sum() == cnt, "an owner collects exactly its channel's partial sums"
    # every position of the (wide) tile is owned by exactly one lane
    assert h["pitch"] == NB * h["pitch1"] and h["pitch1"] >= 1
    owned = np.zeros(P4, dtype=int)
    for r in range(runs):
        for l in range(64):
            b, p0, nl = lanes[r, l]
            if p0 >= 0:
                assert 0 < l < 63 and b == p0 and nl == (p0 % h["pitch"]) // h["pitch1"]
                assert ((p0 + 3) % h["pitch"]) // h["pitch1"] == nl, "a lane's positions straddle two images"
                owned[p0:p0 + 4] += 1
                # both neighbours hold the adjacent groups
                assert lanes[r, l - 1, 0] == b - 4 and lanes[r, l + 1, 0] == b + 4
    assert (owned == 1).all(), "lane table must own every position once"
    # The kernel takes a wave's first run from the table and finds the lanes' groups of its
    # following runs 62 groups further: same thing for every lane that owns outputs or lends
    # data, and in bounds (window buffer + zeroed tail) for the idle ones.
    max_aoff_words = int(rec_off.max()) // 4 % (NB * ps) + 4 if len(rec_off) else 4
    for wq in range(WQ):
        first = lanes[wq * Q, :, 0].astype(np.int64)
        for q in range(1, Q):
            kernel_base = first + 62 * 4 * q
            table = lanes[wq * Q + q]
            live = (table[:, 1] >= 0)
            live[:-1] |= table[1:, 1] >= 0        # lends to the next lane
            live[1:] |= table[:-1, 1] >= 0        # lends to the previous lane
            assert (kernel_base[live] == table[live, 0]).all(), "runs of a wave are not 62 groups apart"
            assert kernel_base.max() + max_aoff_words + 4 <= (NB * ps) + h["tail_floats"]

    out = np.full((N, M, h["E"] * h["F"]), np.nan)
    xf = x.reshape(N, C, H * W).astype(np.float64)
    buf_floats = h["buf_floats"]
    assert buf_floats == h["n_phases"] * CC * NB * ps + ZF and ZF >= P4 + 16
    lds_len = buf_floats + h["tail_floats"]            # one window buffer plus the zeroed tail
    assert h["lds_bytes"] == max((2 * buf_floats + h["tail_floats"]) * 4 + 2 * h["rec_buf_bytes"],
                                 h["max_regions"] * WQ * Q * 1024) <= 160 * 1024
    assert buf_floats * 4 < (1 << 18)
    pad_off = (buf_floats - ZF) * 4 + 16
    assert threads <= 1024 and h["n_items"] * CC * NB <= 12 * threads
    xflat = x.reshape(-1).astype(np.float64)
    for t in range(h["n_tiles"]):
        for n0 in range(0, N, NB):
            nb = min(NB, N - n0)
            acc = np.zeros((bins, K, runs, 64, 4))
            for ch in range(h["n_chunks"]):
                c0 = 0 if ch == 0 else CC0 + (ch - 1) * CC
                ccur = CC0 if ch == 0 else min(CC, C - c0)
                assert ccur >= 1 and c0 + ccur <= C
                # the frame was zeroed once; the staging items rewrite the words that hold input
                lds = np.zeros(lds_len)
                src = slots[t][:, 0].view(np.int32).astype(np.int64)
                key = slots[t][:, 1]
                # the kernel's tests: a slot in use, an image inside the batch, a channel inside C
                live = (src >= 0) & (src < nb * C * H * W) & ((key >> 18) < ccur)
                where = (key[live] & 0x3FFFF).astype(np.int64)
                assert np.all(where % 4 == 0) and len(set(where.tolist())) == len(where)
                assert where.max(initial=0) < (buf_floats - ZF) * 4, "staging must not touch the zero stretch"
                gsrc = (n0 * C + c0) * H * W + src[live]
                assert gsrc.max(initial=0) < N * C * H * W, "staging reads past the end of the input"
                lds[where // 4] = xflat[gsrc]
                if h["n_dma"] > 0:
                    # the same chunk staged by the global -> LDS copies: slot 64*j + lane of a
                    # window buffer takes four consecutive input words, or zeros
                    win_slots = (buf_floats - ZF) // 4
                    assert h["n_dma"] == -(-win_slots // 64) and h["VW"] == 4 and h["WW"] == 4
                    dma = plan[h["off_dma"]:h["off_dma"] + 8 * h["n_tiles"] * h["n_dma"] * 64].view(np.int32)
                    dma = dma.reshape(h["n_tiles"], h["n_dma"] * 64, 2)[t][:win_slots]
                    zero = plan[h["off_zero"]:h["off_zero"] + 64]
                    assert not zero.any() and h["off_zero"] % 16 == 0 and h["off_dma"] % 16 == 0
                    assert (dma[win_slots:, 0] < 0).all() if len(dma) > win_slots else True
                    lds2 = np.zeros(lds_len)
                    for sl in np.nonzero((dma[:, 0] >= 0) & (dma[:, 0] < nb * C * H * W) & (dma[:, 1] < ccur))[0]:
                        g0 = (n0 * C + c0) * H * W + int(dma[sl, 0])
                        assert g0 % 4 == 0 and g0 + 4 <= N * C * H * W
                        lds2[4 * sl:4 * sl + 4] = xflat[g0:g0 + 4]
                    assert np.array_equal(lds, lds2), "the two staging tables disagree"
                for b in range(bins):
                    mgi = b // WM
                    assert seg[b, ch, 0] + seg[b, ch, 1:].sum() <= blk[mgi, ch, 1]
                    assert (int(blk[mgi, ch, 1]) + 1) * B * 8 <= h["rec_buf_bytes"]
                    at = (int(blk[mgi, ch, 0]) + int(seg[b, ch, 0])) * B
                    for k in range(K):
                        for cls in range(NCLS):
                            cnt = int(seg[b, ch, 1 + k * NCLS + cls]) * B
                            for j in range(at, at + cnt):
                                off = int(rec_off[j])
                                assert off % 16 == 0
                                if rec_val[j] == 0.0:      # only padding records carry a zero
                                    assert off == pad_off
                                o = off // 4
                                for r in range(runs):
                                    idx = lanes[r, :, 0][:, None] + o + np.arange(4)[None, :]
                                    assert idx.min() >= 0 and idx.max() < lds_len
                                    acc[b, k, r] += float(rec_val[j]) * _window_words(lds[idx], cls)
                            at += cnt
            # channels split over several accumulator rows: the owner adds the lenders' sums
            for b in range(bins):
                for k in range(K):
                    m, mine, first, cnt = rows[b, k]
                    if m < 0 or mine >= 0:
                        continue
                    g0 = (b // WM) * WM
                    for bb in range(g0, g0 + WM):
                        for kk in range(K):
                            if rows[bb, kk, 0] == m and rows[bb, kk, 1] >= 0:
                                assert first <= rows[bb, kk, 1] < first + cnt
                                acc[b, k] += acc[bb, kk]
            d = dst[t]
            for b in range(bins):
                for k in range(K):
                    m = perm[b, k]
                    if m < 0 or rows[b, k, 1] >= 0:
                        continue
                    for r in range(runs):
                        for l in range(64):
                            _, p0, nl = lanes[r, l]
                            if p0 < 0 or nl >= nb:
                                continue
                            for i in range(4):
                                if d[p0 + i] >= 0:
                                    assert np.isnan(out[n0 + nl, m, d[p0 + i]]), "output written twice"
                                    out[n0 + nl, m, d[p0 + i]] = acc[b, k, r, l, i]
    assert not np.isnan(out).any(), "some output element was never written"
    return out.reshape(N, M, h["E"], h["F"])
