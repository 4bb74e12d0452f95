"""GPU parity: the HIP path (through the C-ABI binding) against the CPU oracle, element by
element on the same seeded inputs.  Integer / copy steps are bit-exact; the fp32 convolution is
held to |gpu - oracle| <= 1e-4 * sum|w*x| per output element."""
import itertools

import numpy as np
import pytest

import paper_1802_10280_amd as esc
from paper_1802_10280_amd import workloads as wl

from helpers import (DeviceLayer, assert_within_bound, oracle_full, random_layers_and_tunings, sample_points,
                     seam_points, to_dev)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    esc.lib()   # raises if the HIP library is missing: no fallback


# ------------------------------------------------------------------ pad_in, bit-exact
@pytest.mark.parametrize("N,C,H,W,pad", [(1, 1, 1, 1, 0), (1, 1, 1, 1, 1), (2, 3, 5, 4, 1), (3, 5, 17, 33, 2),
                                         (2, 7, 56, 56, 1), (1, 2, 300, 7, 3), (4, 9, 13, 13, 0)])
def test_pad_in_bit_exact(oracle, N, C, H, W, pad):
    import torch
    print(f"pad_in N={N} C={C} H={H} W={W} pad={pad}", flush=True)
    rng = np.random.default_rng(N * 100 + C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    x.ravel()[0] = -0.0
    d = esc.make_desc(N, C, H, W, 1, 1, 1, 1, pad)
    d_in = to_dev(x)
    n_pad = esc.escoin_padded_elems(d)
    buf = torch.full((n_pad + 64,), float("nan"), dtype=torch.float32, device="cuda")
    esc.escoin_pad_in(d, d_in, buf[:n_pad])
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    ref = oracle.pad_input(x, pad)
    assert got[:n_pad].tobytes() == ref.tobytes()
    assert np.isnan(got[n_pad:]).all()          # nothing written past the end


# ------------------------------------------------------------------ sconv vs oracle, whole output
SMALL = [
    # N, C, H, W, M, R, S, stride, pad, sparsity
    (1, 1, 3, 3, 1, 3, 3, 1, 0, 0.0),        # single output pixel
    (2, 5, 9, 11, 7, 3, 3, 1, 1, 0.8),
    (3, 16, 14, 14, 32, 3, 3, 1, 1, 0.8),
    (2, 8, 30, 37, 5, 3, 3, 1, 1, 0.6),      # more than one pixel tile, ragged tail
    (2, 6, 33, 35, 4, 3, 3, 2, 1, 0.7),      # stride 2
    (2, 4, 20, 21, 6, 5, 5, 1, 2, 0.7),      # 5x5
    (2, 24, 12, 13, 10, 1, 1, 1, 0, 0.7),    # 1x1 (CSR SpMM)
    (1, 3, 23, 19, 3, 7, 7, 2, 3, 0.5),      # filter size with no specialisation
    (2, 3, 10, 12, 4, 3, 3, 1, 0, 0.5),      # no padding
    (1, 2, 9, 9, 3, 2, 3, 3, 2, 0.3),        # R != S, stride 3
    (2, 12, 13, 13, 9, 3, 3, 1, 1, 0.0),     # dense rows (0 % sparsity)
    (5, 20, 7, 7, 12, 3, 3, 1, 1, 0.8),      # 7x7 maps
    (3, 4, 9, 10, 5, 3, 3, 1, 2, 0.5),       # more padding than the filter needs
    (2, 5, 8, 8, 4, 1, 1, 1, 1, 0.4),        # 1x1 with a frame of zeros (bias-only border)
    (2, 3, 12, 11, 4, 7, 7, 1, 3, 0.6),      # 7x7 stride 1: three shared padding columns
    (3, 4, 9, 9, 5, 4, 4, 1, 1, 0.5),        # even filter: reaches further right than left
    (9, 6, 5, 6, 7, 3, 3, 1, 1, 0.5),        # many small images side by side in one tile
    (5, 6, 11, 1, 10, 4, 1, 1, 3, 0.0),      # one input column, output rows wider than W + pad
]


PATHS = ["direct", "tiled"]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: "x".join(map(str, c)))
def test_sconv_matches_oracle_small(oracle, cfg, path):
    print("sconv small", path, cfg, flush=True)
    N, C, H, W, M, R, S, stride, pad, sp = cfg
    L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, sp, seed=sum(cfg[:9]) + 1, dist="normal")
    dl = DeviceLayer(esc, L)
    for flags in (0, esc.F_BIAS | esc.F_RELU):
        got = dl.run(path, flags)
        ref, bound = oracle_full(oracle, L, flags)
        assert_within_bound(got, ref, bound, f"{path} {cfg} flags={flags}")


def test_random_layers_and_tilings(oracle):
    """The seeded random layers and knobs whose plans the CPU suite replays (there with every
    staged read checked against the bounds of the input): both kernels against the oracle."""
    done = 0
    for L, tune in random_layers_and_tunings(wl, 20260, 90):
        print("sconv random", L.spec, tune, flush=True)
        ref, bound = oracle_full(oracle, L, esc.F_BIAS)
        try:
            dl = DeviceLayer(esc, L, tuning=tune)
            got = dl.forward_tiled(esc.F_BIAS)
        except esc.EscoinError as e:
            assert e.code in (esc.ERANGE, esc.EINVAL), (L.spec, tune)   # a tiling that cannot be realised
            continue
        assert_within_bound(got, ref, bound, f"tiled {L.spec} {tune}")
        assert_within_bound(dl.run("direct", esc.F_BIAS), ref, bound, f"direct {L.spec}")
        done += 1
    assert done >= 70


TUNINGS = [
    dict(K=2, Q=1, B=4, WM=2, CC=3, TH=5),
    dict(K=4, Q=2, B=2, WM=1, CC=2, NB=2),
    dict(K=2, Q=1, B=2, WM=3, CC=5, TH=3),
    dict(K=8, Q=1, B=4, WM=2, CC=1, TH=11),
    dict(K=4, Q=2, B=2, WM=4, CC=7, NB=3),
    dict(K=2, Q=2, B=4, WM=2, CC=6, TH=6),
    dict(K=2, Q=2, B=4, WM=16, CC=2, TH=2),
    dict(K=4, Q=1, B=4, WM=5, CC=4, TH=4),
    dict(K=1, Q=1, B=2, WM=4, CC=2, CS=3),          # channels split over 3 workgroups, atomics
    dict(K=2, Q=2, B=2, WM=2, CC=1, CS=2, TH=7),
    dict(K=1, Q=1, B=2, WM=3, CC=4, NB=3),          # 16-byte staging runs across channels where C % 4 == 0
    dict(K=2, Q=2, B=2, WM=2, CC=8, NB=2),
    dict(K=2, Q=1, B=2, WM=4, WS=2, CC=3, TH=5),            # every channel split over two waves, sums meet in LDS
    dict(K=4, Q=2, B=2, WM=4, WS=4, CC=4, CC0=2, NB=2),     # four ways, short first chunk
    dict(K=1, Q=2, B=2, WM=6, WS=3, CC=5, CC0=1),
    dict(K=2, Q=2, B=2, WM=4, WS=2, CC=2, CS=2),            # split over waves and over workgroups
    dict(K=8, Q=1, B=2, WM=2, WS=2, CC=3, CC0=1, TH=4),
]


@pytest.mark.parametrize("tune", TUNINGS, ids=lambda t: "-".join(f"{k}{v}" for k, v in t.items()))
@pytest.mark.parametrize("cfg", [SMALL[1], SMALL[3], SMALL[4], SMALL[5], SMALL[6], SMALL[11]],
                         ids=lambda c: "x".join(map(str, c)))
def test_tiled_every_template_and_tiling(oracle, cfg, tune):
    """Every kernel instantiation family and odd tilings (bands that do not divide E, chunks
    that do not divide C, several images per workgroup, ragged last image group)."""
    print("sconv tiled tuning", cfg, tune, flush=True)
    N, C, H, W, M, R, S, stride, pad, sp = cfg
    L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, sp, seed=sum(cfg[:9]) + 2, dist="normal")
    t = dict(tune)
    flags = esc.F_BIAS | (esc.F_RELU if "CS" in t else 0)   # the split path clamps in a pass of its own
    try:
        dl = DeviceLayer(esc, L, tuning=t)
        got = dl.forward_tiled(flags)
    except esc.EscoinError as e:
        assert e.code == esc.ERANGE       # a tiling that needs more than 16 waves or too much LDS
        pytest.skip("tiling not realisable for this shape")
    REALISED.add(TUNINGS.index(tune))
    ref, bound = oracle_full(oracle, L, flags)
    assert_within_bound(got, ref, bound, f"{cfg} {tune}")
    if "CS" in t:  # a second call must clear the first call's sums before adding to them
        assert_within_bound(dl.forward_tiled(flags), ref, bound, f"{cfg} {tune} again")


REALISED = set()


def test_every_tuning_was_realised_on_some_shape():
    """Runs after the tuning sweep above: a tiling that no shape could realise would be untested."""
    assert REALISED == set(range(len(TUNINGS))), sorted(set(range(len(TUNINGS))) - REALISED)


@pytest.mark.parametrize("path", PATHS)
def test_non_finite_inputs_stay_where_the_definition_puts_them(oracle, path):
    """An Inf or NaN in the input may only reach the outputs whose window holds it under a
    nonzero weight: records that merely fill a batch, idle lanes and the zero frame must not
    spread it."""
    print("sconv non-finite input", path, flush=True)
    L = wl.custom_layer(3, 7, 12, 13, 9, 3, 3, 1, 1, 0.7, seed=99, dist="normal")
    L.input[1, 2, 5, 6] = np.inf
    L.input[2, 0, 0, 0] = np.nan
    L.input[0, 6, 11, 12] = -np.inf
    for tune in (None, dict(K=2, Q=2, B=2, WM=4, WS=2, CC=3, CC0=1, NB=2)) if path == "tiled" else (None,):
        got = DeviceLayer(esc, L, tuning=tune).run(path, 0)
        with np.errstate(invalid="ignore", over="ignore"):
            ref, bound = oracle_full(oracle, L, 0)
        bad_ref = ~np.isfinite(ref)
        assert bad_ref.any() and (bad_ref == ~np.isfinite(got)).all(), (path, tune, bad_ref.sum(), (~np.isfinite(got)).sum())
        ok = ~bad_ref
        assert (np.abs(got[ok] - ref[ok]) <= 1e-4 * bound[ok]).all()


@pytest.mark.parametrize("path", PATHS)
def test_tiny_config_all_flag_combinations(oracle, path):
    print("sconv T1 flags", path, flush=True)
    L = wl.make_layer("T1")
    dl = DeviceLayer(esc, L)
    pad_ref = oracle.pad_input(L.input, L.spec.pad)
    assert dl.pad().cpu().numpy().tobytes() == pad_ref.tobytes()
    for flags in (0, esc.F_BIAS, esc.F_RELU, esc.F_BIAS | esc.F_RELU):
        got = dl.run(path, flags)
        ref, bound = oracle_full(oracle, L, flags)
        assert_within_bound(got, ref, bound, f"T1 flags={flags}")
        if flags & esc.F_RELU:
            assert (got >= 0).all()


@pytest.mark.parametrize("path", PATHS)
def test_identity_filter_reproduces_input_bit_exact(path):
    """A single centre weight of 1 per output channel copies an input channel exactly."""
    print("sconv identity", path, flush=True)
    rng = np.random.default_rng(1)
    N, C, H, W, M = 2, 6, 15, 17, 6
    w = np.zeros((M, C, 3, 3), dtype=np.float32)
    for m in range(M):
        w[m, (m * 5) % C, 1, 1] = 1.0
    rowptr, colidx, value = wl.dense_to_csr(w)
    spec = wl.LayerSpec("ident", 9, 0, N, C, H, W, M, 3, 3, 1, 1, 0.0)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    L = wl.Layer(spec, w, rowptr, colidx, value, x, np.zeros(M, dtype=np.float32))
    got = DeviceLayer(esc, L).run(path, 0)
    for m in range(M):
        assert got[:, m].tobytes() == x[:, (m * 5) % C].tobytes()


@pytest.mark.parametrize("path", PATHS)
def test_empty_rows_unsorted_rows_and_duplicates(oracle, path):
    print("sconv empty/unsorted/duplicates", path, flush=True)
    L = wl.custom_layer(2, 5, 8, 9, 6, 3, 3, 1, 1, 0.6, seed=4, dist="normal")
    rng = np.random.default_rng(0)
    rows = [list(zip(L.colidx[a:b], L.value[a:b])) for a, b in zip(L.rowptr[:-1], L.rowptr[1:])]
    rows[1] = []                                            # an empty row
    rows[5] = []                                            # last row empty
    rows[2] = rows[2] + [(rows[2][0][0], np.float32(0.25))]  # duplicate entry
    rows[3] = rows[3] + [(7, np.float32(0.0))]              # explicit zero
    for r in rows:
        rng.shuffle(r)                                      # arbitrary order inside each row
    rowptr = np.zeros(7, dtype=np.int32)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.array([c for r in rows for c, _ in r], dtype=np.int32)
    value = np.array([v for r in rows for _, v in r], dtype=np.float32)
    L2 = wl.Layer(L.spec, None, rowptr, colidx, value, L.input, L.bias)
    got = DeviceLayer(esc, L2).run(path, 0)
    ref, bound = oracle_full(oracle, L2, 0)
    assert_within_bound(got, ref, bound, "unsorted")
    assert (got[:, 1] == 0).all() and (got[:, 5] == 0).all()


@pytest.mark.parametrize("path", PATHS)
def test_all_rows_empty_gives_bias_or_zero(oracle, path):
    print("sconv nnz=0", path, flush=True)
    spec = wl.LayerSpec("empty", 9, 0, 2, 3, 6, 6, 4, 3, 3, 1, 1, 1.0)
    rng = np.random.default_rng(2)
    L = wl.Layer(spec, None, np.zeros(5, dtype=np.int32), np.zeros(0, dtype=np.int32),
                 np.zeros(0, dtype=np.float32), rng.random((2, 3, 6, 6), dtype=np.float32),
                 rng.standard_normal(4).astype(np.float32))
    dl = DeviceLayer(esc, L)
    assert (dl.run(path, 0) == 0).all()
    got = dl.run(path, esc.F_BIAS)
    assert (got == L.bias[None, :, None, None]).all()


def test_tiled_buffers_that_are_only_4_byte_aligned(oracle):
    """Input and output that start one float past a 16-byte boundary: the 16-byte output stores
    must give way to 4-byte ones (W and F are multiples of 4 here, so they would be used)."""
    import torch
    print("sconv tiled misaligned buffers", flush=True)
    L = wl.custom_layer(2, 8, 24, 24, 8, 3, 3, 1, 1, 0.6, seed=77, dist="normal")
    dl = DeviceLayer(esc, L)
    ref, bound = oracle_full(oracle, L, esc.F_BIAS)
    assert_within_bound(dl.forward_tiled(esc.F_BIAS), ref, bound, "aligned")
    n_in, n_out = dl.d_in.numel(), dl.d_out.numel()
    big_in = torch.zeros(n_in + 4, dtype=torch.float32, device="cuda")
    big_out = torch.full((n_out + 8,), float("nan"), dtype=torch.float32, device="cuda")
    big_in[1:1 + n_in] = dl.d_in.reshape(-1)
    d_in, d_out = big_in[1:1 + n_in], big_out[1:1 + n_out]
    assert d_out.data_ptr() % 16 == 4
    esc.escoin_sconv_forward_tiled(dl.desc, dl.plan, dl.d_plan, d_in, d_out, dl.d_bias, esc.F_BIAS)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy().reshape(ref.shape)
    assert_within_bound(got, ref, bound, "misaligned")
    assert torch.isnan(big_out[0]) and torch.isnan(big_out[1 + n_out:]).all()   # nothing written outside
    # the aligned call staged by global -> LDS copies, this one word by word through registers:
    # the same sums in the same order
    assert esc.plan_header(dl.plan)["n_dma"] > 0
    assert got.tobytes() == dl.forward_tiled(esc.F_BIAS).tobytes()


def test_small_batch_default_is_one_launch_with_the_same_bits_every_run(oracle):
    """Batch 1: the default plan splits every channel over waves of a workgroup (no atomics), so
    two runs agree bit for bit."""
    print("sconv tiled batch 1 determinism", flush=True)
    L = wl.make_layer("A1b1")
    dl = DeviceLayer(esc, L)
    a = dl.forward_tiled(esc.F_BIAS | esc.F_RELU)
    h = esc.plan_header(dl.plan)
    assert h["CS"] == 1 and h["WS"] > 1 and h["max_regions"] > 0
    for _ in range(3):
        assert dl.forward_tiled(esc.F_BIAS | esc.F_RELU).tobytes() == a.tobytes()


# Shapes outside the bundled workloads, in the plan's default tiling: first layers of the
# paper's networks, 1x1 layers with many channels, large and very wide images.
ODD_SHAPES = [
    # N, C, H, W, M, R, S, stride, pad, sparsity
    (2, 3, 224, 224, 64, 7, 7, 2, 3, 0.5),
    (1, 3, 227, 227, 96, 11, 11, 4, 0, 0.5),
    (2, 64, 56, 56, 256, 1, 1, 1, 0, 0.7),
    (5, 512, 7, 7, 1024, 1, 1, 1, 0, 0.8),
    (2, 32, 112, 112, 32, 3, 3, 1, 1, 0.8),
    (3, 16, 5, 300, 8, 3, 3, 1, 1, 0.6),
    (2, 8, 70, 9, 6, 5, 3, 1, 2, 0.6),
    (70, 4, 3, 3, 5, 3, 3, 1, 1, 0.5),
]


@pytest.mark.parametrize("cfg", ODD_SHAPES, ids=lambda c: "x".join(map(str, c)))
def test_tiled_default_tiling_on_other_shapes(oracle, cfg):
    print("sconv tiled other shapes", cfg, flush=True)
    N, C, H, W, M, R, S, stride, pad, sp = cfg
    L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, sp, seed=sum(cfg[:9]) + 5, dist="normal")
    s = L.spec
    dl = DeviceLayer(esc, L)
    got = dl.forward_tiled(esc.F_BIAS)
    assert np.isfinite(got).all()                       # the buffer was NaN-filled before the call
    pts = sample_points(s, 3000, seed=11)
    Wd = oracle.csr_to_dense(s.M, s.C, s.R, s.S, L.rowptr, L.colidx, L.value)
    ref, bound = oracle.conv_points(L.input, Wd, pts, s.stride, s.pad, bias=L.bias, flags=esc.F_BIAS)
    assert_within_bound(got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, bound, str(cfg))


def test_tiled_random_layers_and_tilings(oracle):
    """Seeded random small layers (filter up to 7x7, strides 1-3, padding 0-3, some with rows of
    whole 16-byte groups) with random knobs and flags; every tiling the plan builder accepts."""
    rng = np.random.default_rng(1802)
    done = 0
    for it in range(200):
        big = rng.random() < 0.3
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        stride, pad = int(rng.choice([1, 1, 1, 2, 3])), int(rng.integers(0, 4))
        H = int(rng.integers(max(1, R - 2 * pad), 40 if big else 20))
        W = int(rng.integers(max(1, S - 2 * pad), 90 if big else 24))
        if rng.random() < 0.4:
            W = max(4, (W // 4) * 4)
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        N = int(rng.integers(1, 3 if big else 12))
        C, M = int(rng.integers(1, 5 if big else 9)), int(rng.integers(1, 6 if big else 12))
        L = wl.custom_layer(N, C, H, W, M, R, S, stride, pad, float(rng.choice([0.0, 0.3, 0.6, 0.9])),
                            seed=9000 + it, dist="normal")
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
        flags = int(rng.integers(0, 4))
        print("sconv tiled random", it, (N, C, H, W, M, R, S, stride, pad), tune, flags, flush=True)
        try:
            got = DeviceLayer(esc, L, tuning=tune or None).forward_tiled(flags)
        except esc.EscoinError as e:
            assert e.code in (esc.ERANGE, esc.EINVAL)
            continue
        ref, bound = oracle_full(oracle, L, flags)
        assert_within_bound(got, ref, bound, f"random case {it}")
        done += 1
    assert done >= 150


def test_tiled_plan_serves_other_batch_sizes(oracle):
    """A plan built for one batch size runs any other: here 8 -> 5 and 8 -> 11 images, with
    several images per tile so that the last tile is ragged."""
    import torch
    print("sconv tiled plan reuse across batch sizes", flush=True)
    L8 = wl.custom_layer(8, 8, 7, 7, 6, 3, 3, 1, 1, 0.6, seed=41, dist="normal")
    d8 = esc.desc_of(L8.spec)
    st = esc.escoin_sconv_pack(d8, L8.rowptr, L8.colidx)
    plan = esc.escoin_sconv_plan_build(d8, L8.rowptr, st, L8.value, esc.make_tuning(NB=3))
    d_plan = to_dev(plan)
    Wd = oracle.csr_to_dense(6, 8, 3, 3, L8.rowptr, L8.colidx, L8.value)
    rng = np.random.default_rng(3)
    for n in (5, 11):
        x = rng.random((n, 8, 7, 7), dtype=np.float32)
        d = esc.make_desc(n, 8, 7, 7, 6, 3, 3, 1, 1)
        d_in = to_dev(x)
        d_out = torch.full((n, 6, 7, 7), float("nan"), dtype=torch.float32, device="cuda")
        esc.escoin_sconv_forward_tiled(d, plan, d_plan, d_in, d_out, None, 0)
        torch.cuda.synchronize()
        ref, bound = oracle.conv(x, Wd, 1, 1)
        assert_within_bound(d_out.cpu().numpy(), ref, bound, f"batch {n}")


# ------------------------------------------------------------------ the paper-shaped layers
# the oracle computes every element of these within seconds: whole output, both entry points
FULL_WHOLE = ["A1b1", "A2b1", "A3b1", "R56", "R28", "R14", "R7", "R56s2", "C56", "G1", "G3", "G5", "S90", "S95"]
# the largest ones: sampled outputs plus every seam of the tiling
FULL_SAMPLED = ["A2b64", "S80", "S80skew", "S80skewperm", "S50", "S70"]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("name", FULL_WHOLE)
def test_full_size_layers_whole_output(oracle, name, path):
    """The bench's layers at the bench's sizes and launch configuration, every output element."""
    print("sconv full", name, path, flush=True)
    L = wl.make_layer(name)
    s = L.spec
    dl = DeviceLayer(esc, L)
    flags = esc.F_BIAS | esc.F_RELU
    got = dl.run(path, flags)
    if path == "direct":
        assert dl.d_padded.cpu().numpy().tobytes() == oracle.pad_input(L.input, s.pad).tobytes()
    ref, bound = oracle_full(oracle, L, flags)
    assert_within_bound(got, ref, bound, name)
    del ref, bound
    if name in ("R56", "R7", "A2b1"):         # once more without the epilogue
        ref, bound = oracle_full(oracle, L, 0)
        assert_within_bound(dl.run(path, 0), ref, bound, name + " plain")


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("name", FULL_SAMPLED)
def test_full_size_layers_sampled_outputs(oracle, name, path):
    """Where the whole output would take the oracle too long: 100 000 random output elements,
    every element on a seam of the tiling, the padded array in full (bit-exact), no unwritten
    element, and the all-ones row-sum property over the whole output."""
    print("sconv full sampled", name, path, flush=True)
    L = wl.make_layer(name)
    s = L.spec
    dl = DeviceLayer(esc, L)
    flags = esc.F_BIAS | esc.F_RELU
    got = dl.run(path, flags)
    assert np.isfinite(got).all()
    if path == "direct":
        pad_ref = oracle.pad_input(L.input, s.pad)
        assert dl.d_padded.cpu().numpy().tobytes() == pad_ref.tobytes()
        del pad_ref
        plan_info = esc.plan_header(esc.escoin_sconv_plan_build(dl.desc, L.rowptr, dl.stretched, L.value))
    else:
        plan_info = esc.plan_header(dl.plan)
    pts = np.concatenate([sample_points(s, 100_000, seed=s.seed), seam_points(s, plan_info, seed=s.seed + 1)])
    Wd = oracle.csr_to_dense(s.M, s.C, s.R, s.S, L.rowptr, L.colidx, L.value)
    ref, bound = oracle.conv_points(L.input, Wd, pts, s.stride, s.pad, bias=L.bias, flags=flags)
    g = got[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    assert_within_bound(g, ref, bound, name)
    # whole-output property that holds at any size: an all-ones input turns every interior
    # output into the CSR row sum
    dl.d_in.fill_(1.0)
    got1 = dl.run(path, 0)
    rowsum = np.array([L.value[a:b].astype(np.float64).sum() for a, b in zip(L.rowptr[:-1], L.rowptr[1:])])
    rowabs = np.array([np.abs(L.value[a:b]).astype(np.float64).sum() for a, b in zip(L.rowptr[:-1], L.rowptr[1:])])
    k = -(-s.pad // s.stride)                              # outputs whose window touches the frame
    inner = got1[:, :, k:s.E - k, k:s.F - k] if k else got1
    err = np.abs(inner - rowsum[None, :, None, None])
    assert (err <= 1e-4 * rowabs[None, :, None, None] + 1e-30).all(), name


# ------------------------------------------------------------------ layers chained on the device
def _chain_check(oracle, layers, tunings=None):
    """Runs the layers back to back on the device, each output (bias + ReLU fused) being the
    next layer's input with nothing in between, and compares the last output with the oracle
    applied layer by layer.  The bound is composed: a layer's own 1e-4 * sum|w*x| plus what the
    deviation allowed on its input can grow to, sum|w| * tol_in (ReLU does not enlarge it)."""
    import torch
    from paper_1802_10280_amd.runner import LayerRunner
    flags = esc.F_BIAS | esc.F_RELU
    runners, x_ref, tol = [], layers[0].input.astype(np.float64), None
    for i, L in enumerate(layers):
        s = L.spec
        runners.append(LayerRunner(L, path="tiled", flags=flags, tuning=(tunings or {}).get(i),
                                   d_in=runners[-1].d_out if i else None))
        Wd = oracle.csr_to_dense(s.M, s.C, s.R, s.S, L.rowptr, L.colidx, L.value)
        x32 = x_ref.astype(np.float32)          # the oracle takes fp32 input, as the device does
        y, bound = oracle.conv(x32, Wd, s.stride, s.pad, bias=L.bias, flags=flags)
        own = 1e-4 * bound + np.abs(x_ref - x32).max() * np.abs(Wd).sum()   # + rounding of the fp32 hand-over
        if tol is not None:
            grown, _ = oracle.conv(tol.astype(np.float32), np.abs(Wd), s.stride, s.pad)
            own = own + grown * (1 + 1e-6)
        x_ref, tol = y, own
    for r in runners:
        r.run()
    torch.cuda.synchronize()
    got = runners[-1].d_out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all() and (got >= 0).all()
    err = np.abs(got - x_ref)
    assert (err <= tol).all(), (err.max(), float((err / np.maximum(tol, 1e-30)).max()))
    # the intermediate maps were really written by the layers before: each equals its own run
    assert float(np.abs(got).max()) > 0
    return float((err / np.maximum(tol, 1e-30)).max())


def test_two_and_three_layers_chained_small(oracle):
    print("sconv chain small", flush=True)
    a = wl.custom_layer(3, 6, 20, 22, 10, 3, 3, 1, 1, 0.6, seed=301, dist="normal")
    b = wl.custom_layer(3, 10, 20, 22, 8, 3, 3, 2, 1, 0.5, seed=302, dist="normal")
    c = wl.custom_layer(3, 8, 10, 11, 12, 1, 1, 1, 0, 0.5, seed=303, dist="normal")
    _chain_check(oracle, [a, b])
    _chain_check(oracle, [a, b, c], tunings={0: dict(K=2, Q=2, TH=7, CC=4), 1: dict(K=2, WM=4, WS=2)})


def test_three_layers_chained_at_bench_size(oracle):
    """The chain the bench times as `--workload chain`: C56 -> R56s2 (stride 2) -> R28 at batch
    32, every output element of the last layer checked."""
    print("sconv chain C56 -> R56s2 -> R28", flush=True)
    _chain_check(oracle, [wl.make_layer(n) for n in wl.CONFIG_LAYERS["chain"]])
