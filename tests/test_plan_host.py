"""CPU checks of the tiled-kernel plan: the blob is replayed by a numpy emulation of the
kernel's data flow and must reproduce the oracle (so table / offset / segment bugs surface
without a GPU), plus the error paths of the plan calls."""
import numpy as np
import pytest

import paper_1802_10280_amd as esc
from paper_1802_10280_amd import workloads as wl

from helpers import random_layers_and_tunings
from plan_sim import simulate

CASES = [
    # (N, C, H, W, M, R, S, stride, pad, sparsity), tuning
    ((2, 5, 9, 11, 7, 3, 3, 1, 1, 0.6), {}),
    ((3, 6, 7, 7, 10, 3, 3, 1, 1, 0.7), dict(K=4, NB=2, CC=4)),
    ((2, 4, 20, 21, 6, 5, 5, 1, 2, 0.7), dict(K=2, TH=5, CC=3)),
    ((2, 6, 17, 19, 5, 3, 3, 2, 1, 0.6), dict(K=4, TH=4, WM=2)),
    ((2, 9, 12, 13, 10, 1, 1, 1, 0, 0.6), dict(K=8, CC=4)),
    ((1, 3, 23, 19, 3, 7, 7, 2, 3, 0.5), dict(K=2, TH=3)),
    ((2, 3, 10, 12, 4, 2, 3, 3, 2, 0.4), dict(K=4, Q=2, B=2)),
    ((5, 8, 7, 7, 12, 3, 3, 1, 1, 0.8), dict(K=8, NB=3, WM=1)),
    ((2, 3, 30, 37, 4, 3, 3, 1, 0, 0.5), dict(TH=6, Q=2)),
    ((7, 5, 7, 7, 6, 3, 3, 1, 1, 0.6), dict(K=2, NB=3)),          # idle lanes between images
    ((6, 4, 13, 13, 5, 3, 3, 1, 1, 0.6), dict(K=2, Q=2, NB=2)),   # two runs, two images
    ((1, 12, 13, 13, 9, 3, 3, 1, 1, 0.6), dict(K=1, CC=2, CS=3)),   # channel chunks dealt to 3 workgroups
    ((3, 4, 9, 10, 5, 3, 3, 1, 2, 0.5), {}),                         # more padding than the filter needs
    ((2, 5, 8, 8, 4, 1, 1, 1, 1, 0.4), dict(NB=2)),                  # 1x1 with a frame of zeros
    ((2, 3, 12, 11, 4, 7, 7, 1, 3, 0.6), {}),                        # 7x7 stride 1
    ((3, 4, 9, 9, 5, 4, 4, 1, 1, 0.5), dict(NB=3)),                  # even filter
    ((9, 6, 5, 6, 7, 3, 3, 1, 1, 0.5), dict(NB=4)),                  # four images side by side, ragged last group
    ((5, 3, 6, 5, 4, 3, 3, 2, 1, 0.5), dict(NB=2)),                  # stride 2 with two images per tile
    ((5, 6, 11, 1, 10, 4, 1, 1, 3, 0.0), dict(CC=3, NB=3)),          # output rows wider than W + pad
    ((6, 8, 7, 7, 9, 3, 3, 1, 1, 0.6), dict(K=1, NB=4, CC=4)),       # 16-byte staging runs across channels
    ((3, 12, 13, 13, 7, 3, 3, 1, 1, 0.6), dict(K=2, Q=2, NB=2, CC=8)),  # the same with a shorter last chunk
    ((2, 5, 9, 11, 7, 3, 3, 1, 1, 0.6), dict(K=2, WM=4, WS=2)),         # every channel split over two waves
    ((3, 6, 7, 7, 10, 3, 3, 1, 1, 0.7), dict(K=4, NB=2, CC=4, WM=4, WS=4, CC0=2)),  # four ways, short first chunk
    ((2, 6, 17, 19, 5, 3, 3, 2, 1, 0.6), dict(K=1, WM=3, WS=3, CC=4, CC0=1)),        # stride 2, three ways
    ((4, 8, 7, 7, 6, 3, 3, 1, 1, 0.5), dict(K=2, Q=2, NB=4, WM=6, WS=3, CC=4, CC0=4, CS=2)),  # split waves and workgroups
    # chunks of more than 256 channels: the staging key must keep the whole channel number
    ((1, 1501, 2, 2, 2048, 1, 1, 1, 0, 0.99), {}),
    ((2, 700, 2, 2, 8, 1, 1, 1, 0, 0.9), dict(CC=400, CS=1)),
    ((30, 1500, 1, 1, 2048, 1, 1, 1, 0, 0.999), dict(NB=1)),
]


@pytest.mark.parametrize("cfg,tune", CASES, ids=lambda c: "x".join(map(str, c)) if isinstance(c, tuple) else str(c))
def test_plan_replay_matches_oracle(oracle, cfg, tune):
    N, C, H, W, M, R, S, stride, pad, sp = cfg
    L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, sp, seed=sum(cfg[:9]) + 3)
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
    plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value, esc.make_tuning(**tune))
    h = esc.plan_header(plan)
    assert h["total_bytes"] == plan.nbytes and h["nnz"] == L.nnz
    for k, v in tune.items():
        assert h[k] == v, (k, h[k], v)
    if C > 256 and not tune.get("CC"):
        assert h["CC"] > 256                     # the case the 8-bit channel field could not hold
    if cfg[:4] in ((6, 8, 7, 7), (3, 12, 13, 13)):
        assert h["VW"] == 4                      # the flat (channel, row, column) runs
    got = simulate(plan, L.input, M)
    Wd = oracle.csr_to_dense(M, C, R, S, L.rowptr, L.colidx, L.value)
    ref, bound = oracle.conv(L.input, Wd, stride, pad)
    assert np.all(np.abs(got - ref) <= 1e-6 * bound + 1e-12)


def test_random_layers_and_tilings_replay(oracle):
    """Seeded random small layers (any filter size, stride, padding) with random knobs: every
    plan the builder accepts must replay to the oracle's result."""
    done = 0
    for L, tune in random_layers_and_tunings(wl, 20260, 90):
        R, S, C, M, stride, pad = L.spec.R, L.spec.S, L.spec.C, L.spec.M, L.spec.stride, L.spec.pad
        d = esc.desc_of(L.spec)
        st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
        try:
            plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value, esc.make_tuning(**tune))
        except esc.EscoinError as e:
            assert e.code in (esc.ERANGE, esc.EINVAL), (L.spec, tune)   # a tiling that cannot be realised
            continue
        got = simulate(plan, L.input, M)
        Wd = oracle.csr_to_dense(M, C, R, S, L.rowptr, L.colidx, L.value)
        ref, bound = oracle.conv(L.input, Wd, stride, pad)
        assert np.all(np.abs(got - ref) <= 1e-6 * bound + 1e-12), (L.spec, tune)
        done += 1
    assert done >= 70


def test_plan_accepts_unsorted_rows_and_duplicates(oracle):
    L = wl.custom_layer(2, 6, 8, 9, 5, 3, 3, 1, 1, 0.5, seed=12)
    rng = np.random.default_rng(1)
    rows = [list(zip(L.colidx[a:b], L.value[a:b])) for a, b in zip(L.rowptr[:-1], L.rowptr[1:])]
    rows[0] = []
    rows[2].append((rows[2][0][0], np.float32(0.5)))
    for r in rows:
        rng.shuffle(r)
    rowptr = np.zeros(6, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c, _ in r], dtype=np.int32)
    value = np.array([v for r in rows for _, v in r], dtype=np.float32)
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, rowptr, colidx)
    plan = esc.escoin_sconv_plan_build(d, rowptr, st, value, esc.make_tuning(K=2, CC=2))
    got = simulate(plan, L.input, 5)
    ref, bound = oracle.conv(L.input, oracle.csr_to_dense(5, 6, 3, 3, rowptr, colidx, value), 1, 1)
    assert np.all(np.abs(got - ref) <= 1e-6 * bound + 1e-12)


def test_long_rows_are_split_over_waves(oracle):
    """One CSR row far longer than a wave's fair share (here: dense, next to rows of a few
    nonzeros) is split over several waves of its workgroup, whose partial sums meet in LDS."""
    rng = np.random.default_rng(5)
    N, C, H, W, M = 2, 16, 9, 9, 12
    w = np.where(rng.random((M, C, 3, 3)) < 0.04, rng.standard_normal((M, C, 3, 3)), 0.0).astype(np.float32)
    w[3] = rng.standard_normal((C, 3, 3)).astype(np.float32)          # 144 nonzeros; the others about 6
    w[7, :8] = rng.standard_normal((8, 3, 3)).astype(np.float32)      # 72
    rowptr, colidx, value = wl.dense_to_csr(w)
    x = rng.random((N, C, H, W), dtype=np.float32)
    d = esc.make_desc(N, C, H, W, M, 3, 3, 1, 1)
    st = esc.escoin_sconv_pack(d, rowptr, colidx)
    for tune in (dict(K=2, WM=8, CC=4, WS=1), dict(K=1, WM=16, CC=16, WS=1), dict(K=4, WM=4, CC=5, WS=2)):
        plan = esc.escoin_sconv_plan_build(d, rowptr, st, value, esc.make_tuning(**tune))
        h = esc.plan_header(plan)
        bins = h["n_mgroups"] * h["WM"]
        rows = plan[h["off_perm"]:h["off_perm"] + 16 * bins * h["K"]].view(np.int32).reshape(-1, 4)
        n_rows_of = np.bincount(rows[rows[:, 0] >= 0, 0], minlength=M)
        assert n_rows_of[3] > max(2, tune.get("WS", 1)) and n_rows_of[3] > n_rows_of[0], (tune, n_rows_of)
        assert h["max_regions"] >= n_rows_of[3] - 1
        # the longest share of any accumulator row stays near a wave's fair share
        nnz_row = np.diff(rowptr)
        share = nnz_row / n_rows_of
        fair = nnz_row.sum() / (h["n_mgroups"] * h["WM"])
        assert share.max() <= max(2.0 * fair, nnz_row.max() / h["WM"] + 1), (tune, share.max(), fair)
        got = simulate(plan, x, M)
        ref, bound = oracle.conv(x, w, 1, 1)
        assert np.all(np.abs(got - ref) <= 1e-6 * bound + 1e-12), tune


def test_explicit_zeros_get_no_record(oracle):
    """An explicit zero in the CSR adds nothing to any sum (the definition skips it); the plan
    gives it no record, so it cannot turn a non-finite input into NaN either."""
    L = wl.custom_layer(2, 4, 6, 6, 3, 3, 3, 1, 1, 0.5, seed=8)
    value = L.value.copy()
    value[::3] = 0.0
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
    plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, value)
    h = esc.plan_header(plan)
    rec_val = plan[h["off_rec"]:h["off_rec"] + 8 * h["n_records"]].view(np.float32)[1::2]
    assert np.count_nonzero(rec_val) == np.count_nonzero(value)
    got = simulate(plan, L.input, 3)
    ref, bound = oracle.conv(L.input, oracle.csr_to_dense(3, 4, 3, 3, L.rowptr, L.colidx, value), 1, 1)
    assert np.all(np.abs(got - ref) <= 1e-6 * bound + 1e-12)


def test_rows_are_dealt_out_balanced():
    L = wl.make_layer("S80skew", with_input=False)
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
    plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value)
    h = esc.plan_header(plan)
    bins = h["n_mgroups"] * h["WM"]
    perm = plan[h["off_perm"]:h["off_perm"] + 16 * bins * h["K"]].view(np.int32).reshape(bins, h["K"], 4)[:, :, 0]
    nnz_row = np.diff(L.rowptr)
    load = np.array([nnz_row[p[p >= 0]].sum() for p in perm])
    assert load.max() <= 1.45 * load.mean()        # rows alone: max/mean = 5.0
    assert nnz_row.max() / nnz_row.mean() > 4.5


@pytest.mark.parametrize("name,tune", [("R7", {}), ("R7", dict(NB=2)), ("A3b64", dict(Q=2, NB=2)),
                                       ("G3", {}), ("R56s2", {})])
def test_lanes_walk_through_the_lds_banks(name, tune):
    """A 16-byte LDS read is conflict-free when the group numbers (word address / 4) of
    consecutive lanes advance by one modulo 16, also across the boundary between two images
    and for the lanes that own nothing."""
    L = wl.make_layer(name, with_input=False)
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
    plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value, esc.make_tuning(**tune))
    h = esc.plan_header(plan)
    runs = h["WQ"] * h["Q"]
    lanes = plan[h["off_lanes"]:h["off_lanes"] + 12 * runs * 64].view(np.int32).reshape(runs, 64, 3)
    assert np.all(lanes[:, :, 0] % 4 == 0)
    group = lanes[:, :, 0] // 4
    for r in range(runs):
        assert len(set((group[r] - np.arange(64)) % 16)) == 1, (name, r)
    assert lanes[:, :, 0].min() == -4 and lanes[:, :, 0].max() <= h["P4"]
    owned = lanes[:, :, 1] >= 0
    assert owned.sum() == h["P4"] // 4                            # every group owned exactly once


def test_plan_error_paths():
    L = wl.custom_layer(1, 4, 8, 8, 4, 3, 3, 1, 1, 0.5, seed=1)
    d = esc.desc_of(L.spec)
    st = esc.escoin_sconv_pack(d, L.rowptr, L.colidx)
    n = esc.escoin_sconv_plan_size(d, L.rowptr, st)
    with pytest.raises(esc.EscoinError) as e:
        esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value, None, np.empty(n - 1, dtype=np.uint8))
    assert e.value.code == esc.ESIZE
    with pytest.raises(esc.EscoinError) as e:        # unstretched column indices are not offsets
        bad = st.copy()
        bad[0] = 3 * 10 + 5                             # r = 3 is outside a 3x3 filter
        esc.escoin_sconv_plan_size(d, L.rowptr, bad)
    assert e.value.code == esc.EINVAL
    with pytest.raises(esc.EscoinError) as e:
        esc.escoin_sconv_plan_size(d, L.rowptr, st, esc.make_tuning(K=3))
    assert e.value.code == esc.EINVAL
    with pytest.raises(esc.EscoinError) as e:        # window does not fit LDS
        big = wl.LayerSpec("big", 9, 0, 1, 64, 200, 200, 4, 3, 3, 1, 1, 0.5)
        esc.escoin_sconv_plan_size(esc.desc_of(big), np.zeros(5, dtype=np.int32), np.zeros(0, dtype=np.int32),
                                   esc.make_tuning(TH=200, CC=64))
    assert e.value.code == esc.ERANGE
    # the forward call rejects a plan built for another geometry before touching the GPU
    plan = esc.escoin_sconv_plan_build(d, L.rowptr, st, L.value)
    other = esc.make_desc(1, 4, 9, 8, 4, 3, 3, 1, 1)
    import ctypes
    one = ctypes.c_void_p(256)
    rc = esc.lib().escoin_sconv_forward_tiled(ctypes.byref(other), plan.ctypes.data, one, one, one, None, 0, None)
    assert rc == esc.EINVAL
    junk = np.zeros(plan.nbytes, dtype=np.uint8)
    rc = esc.lib().escoin_sconv_forward_tiled(ctypes.byref(d), junk.ctypes.data, one, one, one, None, 0, None)
    assert rc == esc.EINVAL
