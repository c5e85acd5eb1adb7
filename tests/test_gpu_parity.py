"""Parity of the HIP path (through the C ABI) with the CPU oracle.

Levels and every packed integer array: bit-exact.  Activations: max abs error
<= 1e-5 against the fp64-accumulating oracle (the bar the task states), and a
much tighter bound in the default (fp64 accumulate) mode where the two differ
only by the rounding of the final store.
"""
import numpy as np
import pytest

import oracle
from workloads import make_config, layered_skip

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5            # the stated bar
TIGHT = 2.5e-7        # default mode: a few float ulps at 1.0


def _amd():
    import paper_2005_04347_amd as amd
    amd.load()
    return amd


@pytest.fixture(scope="module")
def amd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return _amd()


def expected_pack(wl, level, n_levels, heavy=256, medium=32):
    """Host-side statement of what asnn_pack_csr must produce (numpy only)."""
    n = wl.n_nodes
    indeg = np.bincount(wl.dst, minlength=n)
    key = 3 * level.astype(np.int64) + np.where(indeg >= heavy, 0, np.where(indeg >= medium, 1, 2))
    mean = wl.src.shape[0] // n
    full_key = key * 2 + ((indeg < medium) & (4 * indeg <= 3 * mean))     # short light rows end their level
    perm = np.argsort(full_key, kind="stable").astype(np.int32)
    inv = np.empty(n, dtype=np.int32)
    inv[perm] = np.arange(n, dtype=np.int32)
    level_ptr = np.searchsorted(key[perm], np.arange(3 * n_levels + 1), side="left").astype(np.int32)
    row_ptr = np.concatenate([[0], np.cumsum(indeg[perm])]).astype(np.int32)
    order = np.argsort(inv[wl.dst], kind="stable")
    col = inv[wl.src[order]]
    w = wl.w[order]
    return perm, inv, level_ptr, row_ptr, col, w


LEVELS, DATAFLOW, WORKGROUP = 4, 8, 16      # ASNN_FLAG_LEVEL_LAUNCHES, ASNN_FLAG_DATAFLOW, ASNN_FLAG_WORKGROUP
SCHEDULES = [LEVELS, DATAFLOW, WORKGROUP]


def run_gpu(amd, wl, flags=0, poison=True, X=None, net=None):
    """One activation on a NaN-poisoned V (a row read before it is written shows up as NaN)."""
    if net is None:
        net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    X = wl.X if X is None else X
    V = torch.full((wl.n_nodes, X.shape[1]), float("nan"), device="cuda:0") if poison else None
    V, Y = net.activate(X, V=V, flags=flags)
    net.check(X.shape[1])            # synchronises; raises if a dataflow wait gave up
    return net, V, Y


def expected_units(level_ptr, n_levels, row_ptr):
    """numpy statement of the work units: light rows in groups of 16 (never across a level
    boundary), medium rows alone or, in levels of 256 or more of them, in groups of 4, a heavy row of in-degree d in ceil(d / len) chunks of
    len = max(512, ceil(d / 16)) connections, one unit each, all naming the row."""
    starts = []
    first_unit = None
    for k in range(3 * n_levels):
        if k == 3:
            first_unit = len(starts)
        if k % 3 == 0:
            for r in range(level_ptr[k], level_ptr[k + 1]):
                d = int(row_ptr[r + 1] - row_ptr[r])
                length = max(512, -(-d // 16))
                starts += [r] * max(1, -(-d // length))
        else:
            step = 16 if k % 3 == 2 else (4 if level_ptr[k + 1] - level_ptr[k] >= 256 else 1)
            starts += list(range(level_ptr[k], level_ptr[k + 1], step))
    if first_unit is None:
        first_unit = len(starts)
    return np.array(starts + [level_ptr[-1]], dtype=np.int32), first_unit


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_small_configs_levels_pack_activation(amd, idx):
    wl = make_config(idx, "small")
    net, V, Y = run_gpu(amd, wl)
    lv_o, nl_o = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    lv = net.level.cpu().numpy()
    assert net.n_levels == nl_o
    assert (lv == lv_o).all()
    if wl.planted_level is not None:
        assert (lv == wl.planted_level).all()
    g = net.graph
    perm, inv, level_ptr, row_ptr, col, w = expected_pack(wl, lv_o, nl_o)
    assert (g.perm.cpu().numpy() == perm).all()
    assert (g.inv_perm.cpu().numpy() == inv).all()
    assert (g.level_ptr.cpu().numpy() == level_ptr).all()
    assert (g.level_ptr_host == level_ptr).all()
    assert (g.row_ptr.cpu().numpy() == row_ptr).all()
    assert (g.col.cpu().numpy() == col).all()
    assert (g.w.cpu().numpy() == w).all()
    units, first_unit = expected_units(level_ptr, nl_o, row_ptr)
    assert g.n_units == len(units) - 1 and g.first_unit == first_unit
    assert (g.unit_ptr.cpu().numpy()[: g.n_units + 1] == units).all()
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    results = []
    for sched in SCHEDULES:
        _, V, Y = run_gpu(amd, wl, flags=sched, net=net)
        got = net.values_original_order(V).cpu().numpy()
        assert np.isfinite(got).all()
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= TIGHT, (sched, err)
        assert (Y.cpu().numpy() == got[wl.output_ids]).all()
        results.append(got)
        # fp32 accumulation is the fast mode, not the parity mode: with weights in
        # [-2,2] (config 5) or in-degrees in the thousands (config 4) its rounding
        # noise alone exceeds 1e-5 (the oracle's own fp32 variant shows the same).
        _, V32, _ = run_gpu(amd, wl, flags=sched | amd.FLAG_ACC_F32, net=net)
        got32 = net.values_original_order(V32).cpu().numpy()
        err32 = float(np.abs(got32.astype(np.float64) - want).max())
        assert err32 <= (TOL if idx <= 3 else 30 * TOL), (sched, err32)
    assert (results[0] == results[1]).all()          # both schedules give the same bits


@pytest.mark.parametrize("B", [1, 2, 3, 4, 6, 8, 12, 20, 36, 64, 100, 127, 128, 130, 256, 260, 516])
def test_batch_widths_cover_every_lane_layout(amd, B):
    """Every (vector width, lanes-per-tile) kernel variant, ragged tiles included."""
    wl = layered_skip(seed=5, n_nodes=700, n_inputs=19, n_outputs=9, n_levels=7, B=B, mean_extra_degree=9.0)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net = None
    for sched in SCHEDULES:
        net, V, Y = run_gpu(amd, wl, flags=sched, net=net)
        got = net.values_original_order(V).cpu().numpy()
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= TIGHT, (sched, err)
        assert (Y.cpu().numpy() == got[wl.output_ids]).all(), sched
        _, V32, _ = run_gpu(amd, wl, flags=sched | amd.FLAG_ACC_F32, net=net)
        got32 = net.values_original_order(V32).cpu().numpy()
        err32 = float(np.abs(got32.astype(np.float64) - want).max())
        assert err32 <= TOL, (sched, err32)


@pytest.mark.parametrize("rows_per_level", [25, 100])
@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 8, 12, 16, 20, 32, 36])
def test_narrow_levels_in_one_workgroup(amd, B, rows_per_level):
    """The workgroup schedule hands the light rows of a narrow level to teams of 16 lanes (at most 64
    rows, 128 with one column per lane) and walks wider levels one lane group per row: both sides of
    that switch for every lane layout that has teams, with rows of up to 31 connections (more than
    one round for the layouts whose teams hold few lane groups)."""
    n_levels = 9
    n_io = 11
    wl = layered_skip(seed=3 + rows_per_level, n_nodes=2 * n_io + rows_per_level * (n_levels - 2), n_inputs=n_io,
                      n_outputs=n_io, n_levels=n_levels, B=B, mean_extra_degree=15.0)
    indeg = np.bincount(wl.dst, minlength=wl.n_nodes)
    assert ((indeg > 16) & (indeg < 32)).sum() > 20            # light rows that need a second round
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net, V, Y = run_gpu(amd, wl, flags=WORKGROUP)
    got = net.values_original_order(V).cpu().numpy()
    err = float(np.abs(got.astype(np.float64) - want).max())
    assert err <= TIGHT, err
    assert (Y.cpu().numpy() == got[wl.output_ids]).all()
    _, V32, _ = run_gpu(amd, wl, flags=WORKGROUP | amd.FLAG_ACC_F32, net=net)
    err32 = float(np.abs(net.values_original_order(V32).cpu().numpy().astype(np.float64) - want).max())
    assert err32 <= TOL, err32
    _, V2, _ = run_gpu(amd, wl, flags=WORKGROUP, net=net)
    assert torch.equal(V, V2)                                  # the order of the additions is fixed


@pytest.mark.parametrize("B", [1, 3, 8, 32])
def test_narrow_levels_of_a_network_too_large_for_lds(amd, B):
    """The same teams when the workgroup schedule reads the network from global memory (some
    60 000 connections: beyond what a workgroup can stage) and stores each value straight to V."""
    n_levels, n_io, rows_per_level = 150, 9, 30
    wl = layered_skip(seed=11, n_nodes=2 * n_io + rows_per_level * (n_levels - 2), n_inputs=n_io, n_outputs=n_io,
                      n_levels=n_levels, B=B, mean_extra_degree=12.5)
    assert wl.n_edges * 8 > 160 * 1024
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net, V, Y = run_gpu(amd, wl, flags=WORKGROUP)
    got = net.values_original_order(V).cpu().numpy()
    err = float(np.abs(got.astype(np.float64) - want).max())
    assert err <= TIGHT, err
    assert (Y.cpu().numpy() == got[wl.output_ids]).all()
    _, V32, _ = run_gpu(amd, wl, flags=WORKGROUP | amd.FLAG_ACC_F32, net=net)
    err32 = float(np.abs(net.values_original_order(V32).cpu().numpy().astype(np.float64) - want).max())
    assert err32 <= 30 * TOL, err32


@pytest.mark.parametrize("B", [1, 16, 130])
def test_levels_of_many_medium_rows(amd, B):
    """Levels of 256 or more medium rows put them four to a work unit (four wavefronts a row), with
    ragged last units of one, two and three rows; narrower levels keep a unit per row."""
    n_io, n_levels = 40, 8
    sizes = [300, 301, 302, 303, 120, 299]
    wl = layered_skip(seed=21, n_nodes=2 * n_io + sum(sizes), n_inputs=n_io, n_outputs=n_io, n_levels=n_levels, B=B,
                      mean_extra_degree=50.0)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    g = net.graph
    level_ptr = g.level_ptr.cpu().numpy()
    row_ptr = g.row_ptr.cpu().numpy()
    medium = level_ptr[2::3][:n_levels] - level_ptr[1::3][:n_levels]
    assert (medium >= 256).sum() >= 3 and ((medium > 0) & (medium < 256)).sum() >= 1
    assert len({int(m) % 4 for m in medium if m >= 256}) >= 2          # ragged last units
    units, first_unit = expected_units(level_ptr, net.n_levels, row_ptr)
    assert g.n_units == len(units) - 1 and g.first_unit == first_unit
    assert (g.unit_ptr.cpu().numpy()[: g.n_units + 1] == units).all()
    for sched in SCHEDULES:
        _, V, Y = run_gpu(amd, wl, flags=sched, net=net)
        got = net.values_original_order(V).cpu().numpy()
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= TIGHT, (sched, err)
        assert (Y.cpu().numpy() == got[wl.output_ids]).all(), sched


@pytest.mark.parametrize("B", [1, 130])
def test_inputs_and_outputs_in_pinned_host_memory(amd, B):
    """X and Y may live in pinned host memory that the device addresses: every schedule reads the
    inputs and writes the output rows in place, with the bits of the device-resident call."""
    wl = layered_skip(seed=9, n_nodes=500, n_inputs=17, n_outputs=13, n_levels=9, B=B, mean_extra_degree=9.0)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    Xp = torch.empty(wl.X.shape, dtype=torch.float32, pin_memory=True)
    Xp.copy_(torch.from_numpy(wl.X))
    for sched in SCHEDULES:
        _, V, Y = run_gpu(amd, wl, flags=sched, net=net)
        Yp = torch.full((len(wl.output_ids), B), float("nan"), dtype=torch.float32).pin_memory()
        V2 = torch.full((wl.n_nodes, B), float("nan"), device="cuda:0")
        amd.asnn_activate(net.graph, net.input_ids, Xp, net.output_ids, V=V2, Y=Yp, flags=sched, workspace=net.workspace(B))
        net.check(B)
        assert torch.equal(V2, V), sched
        assert torch.equal(Yp, Y.cpu()), sched


@pytest.mark.parametrize("B", [1, 5, 64, 130])
def test_output_rows_of_any_level_and_bad_ids(amd, B):
    """Y takes the rows of output_ids whatever their level: a sensor, a hidden node, a node listed
    twice; an id outside [0, n_nodes) gives a row of NaN.  Every schedule, 20 outputs (more than
    one group of 16 for the schedule that copies them with work items of its own)."""
    wl = layered_skip(seed=11, n_nodes=400, n_inputs=12, n_outputs=5, n_levels=9, B=B, mean_extra_degree=6.0)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    rng = np.random.default_rng(B)
    ids = np.concatenate([wl.output_ids, wl.input_ids[:3], rng.integers(0, wl.n_nodes, size=9), [wl.output_ids[0]],
                          [wl.n_nodes, -1]]).astype(np.int32)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, ids)
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        V, Y = net.activate(wl.X, flags=sched)
        net.check(B)
        y = Y.cpu().numpy()
        got = net.values_original_order(V).cpu().numpy()
        assert np.abs(got.astype(np.float64) - want).max() <= TIGHT
        assert (y[:-2] == got[ids[:-2]]).all(), sched
        assert np.isnan(y[-2:]).all(), sched


def test_required_set_on_a_sorted_adjacency(amd):
    """Networks with millions of connections group them with a sort instead of a counting pass:
    the required set of the 16 M-connection workload, bit-exact, and its levels once more."""
    wl = make_config(4, "full")
    dev = "cuda:0"
    src = torch.from_numpy(wl.src).to(dev); dst = torch.from_numpy(wl.dst).to(dev)
    outs = torch.from_numpy(wl.output_ids[:3]).to(dev)
    req, n_req = amd.asnn_required_set(wl.n_nodes, src, dst, outs)
    want = oracle.required(wl.n_nodes, wl.src, wl.dst, wl.output_ids[:3])
    assert (req.cpu().numpy().astype(bool) == want).all() and n_req == int(want.sum())
    assert 0 < n_req < wl.n_nodes
    level, n_levels = amd.asnn_build_levels(wl.n_nodes, src, dst, torch.from_numpy(wl.input_ids).to(dev))
    lv, nl = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    assert n_levels == nl and (level.cpu().numpy() == lv).all()


def _heavy_workload(B, seed=3):
    """A few rows with in-degree far above the heavy threshold (parallel edges
    included), mixed with light rows and a non-sensor root."""
    rng = np.random.default_rng(seed)
    n_in, n_mid = 300, 60
    n = n_in + 1 + n_mid + 3
    root = n_in                      # zero in-degree, not a sensor
    src, dst = [], []
    for m in range(n_mid):
        d = [1, 7, 31, 32, 33, 100, 255, 256, 257, 512, 513, 900, 4096, 5000, 20000][m % 15]
        src += rng.integers(0, n_in + 1, size=d).tolist()
        dst += [n_in + 1 + m] * d
    for t in range(3):
        d = [3, 600, 2000][t]
        src += rng.integers(0, n_in + 1 + n_mid, size=d).tolist()
        dst += [n_in + 1 + n_mid + t] * d
    src = np.array(src, dtype=np.int32); dst = np.array(dst, dtype=np.int32)
    w = rng.uniform(-1, 1, size=src.shape[0]).astype(np.float32)
    X = rng.uniform(0, 1, size=(n_in, B)).astype(np.float32)
    relabel = rng.permutation(n).astype(np.int32)
    ep = rng.permutation(src.shape[0])
    from workloads import Workload
    return Workload("heavy", n, relabel[src][ep], relabel[dst][ep], w[ep], relabel[np.arange(n_in)],
                    relabel[np.arange(n - 3, n)], X), relabel[root]


@pytest.mark.parametrize("B", [1, 5, 64, 256, 1024])
def test_heavy_rows_and_non_sensor_root(amd, B):
    wl, root = _heavy_workload(B)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net = None
    for sched in SCHEDULES:
        net, V, _ = run_gpu(amd, wl, flags=sched, net=net)
        lp = net.graph.level_ptr_host
        assert lp[4] - lp[3] > 0 and lp[7] - lp[6] > 0          # heavy ranges of levels 1 and 2 are populated
        assert lp[5] - lp[4] > 0 and lp[6] - lp[5] > 0          # and so are the medium and light ones of level 1
        g = net.graph
        units, first_unit = expected_units(lp, net.n_levels, g.row_ptr.cpu().numpy())     # rows cut into 2 .. 16 chunks
        assert g.n_units == len(units) - 1 and g.first_unit == first_unit
        assert (g.unit_ptr.cpu().numpy()[: g.n_units + 1] == units).all()
        assert g.record.max_heavy_indegree == 20000
        got = net.values_original_order(V).cpu().numpy()
        assert (got[root] == np.float32(0.5)).all()
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= TIGHT, (sched, err)
        _, V32, _ = run_gpu(amd, wl, flags=sched | amd.FLAG_ACC_F32, net=net)
        got32 = net.values_original_order(V32).cpu().numpy()
        err32 = float(np.abs(got32.astype(np.float64) - want).max())
        assert err32 <= 30 * TOL, (sched, err32)      # thousands of fp32 terms per sum: fast mode only


def test_deterministic_and_raw_inputs(amd):
    wl = make_config(3, "small")
    net, V1, Y1 = run_gpu(amd, wl, flags=LEVELS)
    for sched in (LEVELS, DATAFLOW, 0, WORKGROUP, DATAFLOW, WORKGROUP):
        V2, Y2 = net.activate(wl.X, flags=sched)
        net.check(wl.B)
        assert torch.equal(V1, V2) and torch.equal(Y1, Y2)
    # without a workspace only level launches are possible; forcing dataflow is refused
    V2, _ = net.activate(wl.X, use_workspace=False)
    torch.cuda.synchronize()
    assert torch.equal(V1, V2)
    with pytest.raises(amd.AsnnError):
        net.activate(wl.X, flags=DATAFLOW, use_workspace=False)
    with pytest.raises(amd.AsnnError):
        net.activate(wl.X, flags=DATAFLOW | WORKGROUP)          # two schedules forced at once
    V2, Y2 = net.activate(wl.X, flags=WORKGROUP, use_workspace=False)      # needs no workspace
    torch.cuda.synchronize()
    assert torch.equal(V1, V2) and torch.equal(Y1, Y2)
    for sched in SCHEDULES:
        V3, _ = net.activate(wl.X, flags=sched | amd.FLAG_RAW_INPUTS)
        net.check(wl.B)
        want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X, raw_inputs=True)
        got = net.values_original_order(V3).cpu().numpy()
        assert np.abs(got.astype(np.float64) - want).max() <= TIGHT
    V3, _ = net.activate(wl.X, flags=amd.FLAG_RAW_INPUTS)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X, raw_inputs=True)
    got = net.values_original_order(V3).cpu().numpy()
    assert np.abs(got.astype(np.float64) - want).max() <= TIGHT


def test_saturation_gives_exact_zero_and_one(amd):
    """4096 parallel connections of weight -1 (and +1) from a 0.5 sensor, and
    huge raw inputs: e^(-4.97x) overflows, the result is exactly 0 / 1."""
    from workloads import Workload
    src = np.zeros(8192, dtype=np.int32)
    dst = np.concatenate([np.full(4096, 1), np.full(4096, 2)]).astype(np.int32)
    w = np.concatenate([np.full(4096, -1.0), np.full(4096, 1.0)]).astype(np.float32)
    for flags in (LEVELS, LEVELS | 2, DATAFLOW, DATAFLOW | 2, WORKGROUP, WORKGROUP | 2):
        wl = Workload("sat", 3, src, dst, w, np.array([0], np.int32), np.array([1, 2], np.int32),
                      np.zeros((1, 4), np.float32))
        _, V, Y = run_gpu(amd, wl, flags=flags)
        y = Y.cpu().numpy()
        assert (y[0] == 0.0).all() and (y[1] == 1.0).all()
    wl = Workload("sat2", 2, np.array([0], np.int32), np.array([1], np.int32), np.array([-1.0], np.float32),
                  np.array([0], np.int32), np.array([1], np.int32),
                  np.array([[30.0, 1000.0, 3.0e38, -3.0e38]], np.float32))
    for flags in (LEVELS | 1, LEVELS | 3, DATAFLOW | 1, DATAFLOW | 3, WORKGROUP | 1, WORKGROUP | 3):
        _, V, Y = run_gpu(amd, wl, flags=flags)
        y = Y.cpu().numpy()[0]
        assert (y[:3] == 0.0).all() and y[3] == 1.0


def test_sigmoid_over_a_dense_range_of_sums(amd):
    """One connection of weight 1 from a raw sensor into a node, for 200 000 sensor values across the
    range where the sigmoid moves and out into both tails: the default mode must give the fp64
    sigmoid rounded to fp32 (the last bit may differ where the fp64 value sits on a rounding
    boundary: at most one float ulp, and rarely), NaN stays NaN, the far tails are exactly 0 and 1."""
    from workloads import Workload
    n = 2000
    B = 100
    rng = np.random.default_rng(5)
    x = np.concatenate([np.linspace(-9.0, 9.0, n * B - 4000), rng.uniform(-200.0, 200.0, 3990),
                        [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-30, -1e-30, 88.0, -88.0, 150.0]]).astype(np.float32)
    x = x.reshape(n, B)
    src = np.arange(n, dtype=np.int32)
    dst = np.arange(n, 2 * n, dtype=np.int32)
    wl = Workload("sigmoid", 2 * n, src, dst, np.ones(n, np.float32), src.copy(), dst.copy(), x)
    with np.errstate(over="ignore"):
        want = (1.0 / (1.0 + np.exp(-4.97 * x.astype(np.float64)))).astype(np.float32)
    for flags in (LEVELS | 1, DATAFLOW | 1, WORKGROUP | 1):
        _, V, Y = run_gpu(amd, wl, flags=flags)
        got = Y.cpu().numpy()
        nan = np.isnan(want)
        assert (np.isnan(got) == nan).all()
        diff = np.abs(got[~nan].astype(np.float64) - want[~nan])
        ulp = np.spacing(want[~nan]).astype(np.float64)
        assert (diff <= ulp).all(), float(diff.max())
        assert (diff > 0).mean() < 1e-4, float((diff > 0).mean())
        assert (got[x > 20] == 1.0).all() and (got[x < -40] == 0.0).all()


def test_degenerate_networks(amd):
    from workloads import Workload
    # no connections at all: sensors squash, the other node gives 0.5
    wl = Workload("noedge", 3, np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                  np.array([2, 0], np.int32), np.array([1, 2], np.int32), np.array([[0.0, 1.0], [0.25, 0.5]], np.float32))
    want = oracle.activate(3, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        net, V, Y = run_gpu(amd, wl, flags=sched)
        assert net.n_levels == 1
        got = net.values_original_order(V).cpu().numpy()
        assert np.abs(got - want).max() <= TIGHT and (got[1] == 0.5).all()
    # a single node, a single chain
    wl = Workload("chain", 5, np.arange(4, dtype=np.int32), np.arange(1, 5, dtype=np.int32),
                  np.array([1.0, -2.0, 0.5, 3.0], np.float32), np.array([0], np.int32), np.array([4], np.int32),
                  np.array([[0.3]], np.float32))
    want = oracle.activate(5, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        net, V, Y = run_gpu(amd, wl, flags=sched)
        assert net.n_levels == 5
        assert np.abs(net.values_original_order(V).cpu().numpy() - want).max() <= TIGHT
    # no sensor at all: every root gives 0.5; no output requested either
    wl = Workload("nosensor", 6, np.array([0, 1, 2, 2, 3], np.int32), np.array([2, 2, 3, 4, 5], np.int32),
                  np.array([1.5, -0.5, 2.0, -2.0, 0.25], np.float32), np.zeros(0, np.int32), np.zeros(0, np.int32),
                  np.zeros((0, 3), np.float32))
    want = oracle.activate(6, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    assert want.shape == (6, 3)
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        net, V, Y = run_gpu(amd, wl, flags=sched)
        got = net.values_original_order(V).cpu().numpy()
        assert np.abs(got - want).max() <= TIGHT and (got[:2] == 0.5).all()


@pytest.mark.parametrize("B", [1, 7, 130])
def test_bad_input_ids_leave_no_root_unwritten(amd, B):
    """asnn_activate takes the input ids as they come: one out of range is skipped, one listed twice
    is staged twice.  With such a list the number of ids can equal the number of rows in level 0
    although the level also holds roots that are no sensors; every such root must still come out
    as sigmoid(0) = 0.5, in every schedule, on a value matrix that arrives full of NaN."""
    wl = layered_skip(seed=13, n_nodes=300, n_inputs=3, n_outputs=5, n_levels=6, B=B, mean_extra_degree=4.0)
    # the network keeps its three roots, but only the first is a sensor
    sensor, roots = wl.input_ids[:1], wl.input_ids[1:]
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, sensor, wl.output_ids)
    lp = net.graph.level_ptr_host
    assert lp[3] == 3                                             # level 0: one sensor, two other roots
    bad = np.array([sensor[0], wl.n_nodes + 5, sensor[0]], dtype=np.int32)      # as many ids as level-0 rows
    X = np.ascontiguousarray(wl.X[[0, 1, 0]])                      # the repeated id gets the same row both times
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, sensor, wl.X[:1])
    ids = torch.from_numpy(bad).cuda()
    Xd = torch.from_numpy(X).cuda()
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        V = torch.full((wl.n_nodes, B), float("nan"), device="cuda:0")
        V, Y = amd.asnn_activate(net.graph, ids, Xd, net.output_ids, V=V, flags=sched, workspace=net.workspace(B))
        net.check(B)
        got = net.values_original_order(V).cpu().numpy()
        assert (got[roots] == np.float32(0.5)).all(), sched
        assert np.abs(got.astype(np.float64) - want).max() <= TIGHT, sched
        assert (Y.cpu().numpy() == got[wl.output_ids]).all(), sched


def test_error_codes_from_device_checks(amd):
    dev = "cuda:0"
    t = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([0, 1, 2]), t([1, 2, 0]), t([]))
    assert e.value.code == -6
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([1]), t([1]), t([0]))
    assert e.value.code == -6
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([0]), t([3]), t([0]))
    assert e.value.code == -3
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([0]), t([1]), t([1]))
    assert e.value.code == -4
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([0]), t([1]), t([0, 0]))
    assert e.value.code == -5
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(3, t([0]), t([1]), t([7]))
    assert e.value.code == -3
    # pack rejects a level array that does not increase along a connection
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_pack_csr(3, 2, t([0, 1]), t([1, 2]), torch.ones(2, device=dev), t([0, 1, 1]))
    assert e.value.code == -9
    lv, nl = amd.asnn_build_levels(0, t([]), t([]), t([]))
    assert nl == 0


def _stages_network(stages, rng):
    """Layered DAG from a list of stage widths; stage s+1 nodes draw their sources from stage s
    (`fan` sources each, or all of stage s when fan is None), plus a few from any earlier stage."""
    src, dst = [], []
    first = [0]
    for width, _ in stages:
        first.append(first[-1] + width)
    for s in range(1, len(stages)):
        width, fan = stages[s]
        lo, hi = first[s - 1], first[s]
        for v in range(first[s], first[s + 1]):
            if fan is None:
                picks = np.arange(lo, hi)
            else:
                picks = rng.integers(lo, hi, size=fan)
                picks[0] = lo + (v % (hi - lo))           # every node of the stage below is used when widths allow
            extra = rng.integers(0, hi, size=2)            # skip connections (and parallel ones)
            for a in np.concatenate([picks, extra]):
                src.append(int(a)); dst.append(v)
    n = first[-1]
    src, dst = np.array(src, np.int32), np.array(dst, np.int32)
    relabel = rng.permutation(n).astype(np.int32)
    order = rng.permutation(len(src))
    return n, relabel[src][order], relabel[dst][order]


@pytest.mark.parametrize("seed", [0, 1])
def test_levels_across_narrow_and_wide_frontiers(amd, seed):
    """Level assignment where the frontier keeps changing regime: narrow layers (swept by one
    workgroup without leaving the device), layers wider than that workgroup keeps (grid-wide
    sweeps), a node with 70000 outgoing connections, nodes with thousands of incoming ones (their
    releases are added up per workgroup first), and back to a long narrow tail.  Bit-exact
    against the oracle."""
    rng = np.random.default_rng(seed)
    stages = [(3, 0), (5, 2), (1, None), (6000, 1), (2, None), (40, 1), (1, None), (70000, 1), (3, None),
              (300, 2), (1, None), (2500, 1), (2048, 3), (2049, 2), (7, 300)]
    stages += [(int(w), 3) for w in rng.integers(1, 60, size=150)]
    n, src, dst = _stages_network(stages, rng)
    want, want_levels = oracle.levels(n, src, dst)
    roots = np.flatnonzero(np.bincount(dst, minlength=n) == 0).astype(np.int32)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    got, n_levels = amd.asnn_build_levels(n, t(src), t(dst), t(roots[:2]))
    assert n_levels == want_levels == len(stages)
    assert np.array_equal(got.cpu().numpy(), want)
    # a cycle inside the narrow tail is still reported
    hi = lo = np.flatnonzero(want == want_levels - 1)[0]
    for _ in range(19):                                   # walk to an ancestor of hi, one level at a time
        into = np.flatnonzero(dst == lo)
        lo = src[into[np.argmax(want[src[into]])]]
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_build_levels(n, t(np.append(src, hi).astype(np.int32)), t(np.append(dst, lo).astype(np.int32)), t(roots[:2]))
    assert e.value.code == -6


@pytest.mark.parametrize("block", [1, 1500])
def test_levels_with_out_degrees_around_the_sweep_batches(amd, block):
    """The grid-wide sweeps release a node's outgoing connections 16 lanes x 4 at a time: out-degrees on
    both sides of every multiple of 16 up to 64 and of 64 beyond, in a random DAG over a topological order
    cut into blocks of `block` nodes, every connection leading into one of the next three blocks (1: thousands
    of layers of a few nodes, the single workgroup's sweeps after a grid-wide start; 1500: a dozen layers of
    some 1500 nodes, grid-wide sweeps throughout).  Bit-exact."""
    rng = np.random.default_rng(17 + block)
    n = 20000
    degrees = np.array([0, 1, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 127, 128, 129, 200, 257])
    src, dst = [], []
    for i in range(n):
        d = int(degrees[rng.integers(0, len(degrees))])
        lo = (i // block + 1) * block
        hi = min(n, lo + 3 * block)
        if d and lo < hi:
            src.append(np.full(d, i, np.int32))
            dst.append(rng.integers(lo, hi, size=d).astype(np.int32))
    src, dst = np.concatenate(src), np.concatenate(dst)
    relabel = rng.permutation(n).astype(np.int32)
    order = rng.permutation(len(src))
    src, dst = relabel[src][order], relabel[dst][order]
    assert len(src) > 1_000_000
    want, want_levels = oracle.levels(n, src, dst)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    got, n_levels = amd.asnn_build_levels(n, t(src), t(dst), t(np.zeros(0, np.int32)))
    assert n_levels == want_levels
    assert np.array_equal(got.cpu().numpy(), want)


def test_levels_of_a_very_deep_network(amd):
    """4500 layers of one to three nodes behind two wide ones: the sweeps change from the grid-wide
    kernel to the single workgroup that runs sweep after sweep on the device, whose count of sweeps is
    only bounded by the network."""
    rng = np.random.default_rng(4)
    stages = [(3000, 0), (2500, 2)] + [(int(w), 2) for w in rng.integers(1, 4, size=4500)]
    n, src, dst = _stages_network(stages, rng)
    want, want_levels = oracle.levels(n, src, dst)
    assert want_levels == len(stages) > 4096
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    got, n_levels = amd.asnn_build_levels(n, t(src), t(dst), t(np.zeros(0, np.int32)))
    assert n_levels == want_levels
    assert np.array_equal(got.cpu().numpy(), want)


def _max_abs_err_every_element(V, inv, want, rows_per_chunk=1 << 18):
    """max |V[inv] - want| over EVERY element, in fp64 (exact for two floats), row chunk by row chunk
    so that the temporaries stay small next to a value matrix of a gigabyte.  V is the device result
    in packed row order, inv maps original ids to packed rows, want is the oracle's host array in
    original ids.  Also returns whether any element of the device result is NaN."""
    worst, any_nan = 0.0, False
    for r0 in range(0, want.shape[0], rows_per_chunk):
        r1 = min(r0 + rows_per_chunk, want.shape[0])
        got = V[inv[r0:r1]].cpu().numpy()
        any_nan = any_nan or bool(np.isnan(got).any())
        worst = max(worst, float(np.abs(got.astype(np.float64) - want[r0:r1]).max()))
    return worst, any_nan


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_full_size_configs(amd, idx):
    """The five workloads at full size, in the default schedule (the one the benchmark times) and
    in every forced schedule.  Levels and packed arrays: every element, bit-exact.  Activations:
    the oracle evaluates ALL batch columns and every element of the value matrix is compared, for
    every schedule (every column tile and both edges of every tile of the kernels' launch
    configuration are covered)."""
    wl = make_config(idx, "full")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    lv = net.level.cpu().numpy()
    lv_o, nl_o = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    assert net.n_levels == nl_o and (lv == lv_o).all()
    if wl.planted_level is not None:
        assert (lv == wl.planted_level).all()
    # the packed arrays, bit for bit (the large workloads take the preprocess paths that sort first)
    perm, inv_np, level_ptr, row_ptr, col, w = expected_pack(wl, lv_o, nl_o)
    g = net.graph
    assert (g.perm.cpu().numpy() == perm).all() and (g.inv_perm.cpu().numpy() == inv_np).all()
    assert (g.level_ptr_host == level_ptr).all() and (g.row_ptr.cpu().numpy() == row_ptr).all()
    assert (g.col.cpu().numpy() == col).all() and (g.w.cpu().numpy() == w).all()
    del perm, inv_np, col, w
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)       # [N, B], every column
    assert want.shape == (wl.n_nodes, wl.B) and np.isfinite(want).all()
    inv = net.graph.inv_perm.long()
    outs = torch.as_tensor(wl.output_ids.astype(np.int64), device="cuda:0")
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        _, V, Y = run_gpu(amd, wl, flags=sched, net=net)
        err, any_nan = _max_abs_err_every_element(V, inv, want)
        print(f"config {idx} schedule {sched} ({amd.asnn_activate_schedule(net.graph, wl.B, True, sched)}): "
              f"N={wl.n_nodes} E={wl.n_edges} B={wl.B} L={nl_o} elements={wl.n_nodes * wl.B} max_abs_err={err:.3e}")
        assert not any_nan, sched
        assert err <= TOL, (sched, err)
        assert torch.equal(Y, V[inv[outs]]), sched
        del V, Y


def test_full_size_benchmark_workload_in_the_fast_mode(amd):
    """The benchmark workload with fp32 sums (ASNN_FLAG_ACC_F32, the mode `bench.py --flags 2` times): every
    element of the value matrix within the same 1e-5 of the oracle, in the level launches and the dataflow
    schedule (the deep and the population workloads do not meet the bound with fp32 sums, which is why
    fp64 sums are the default and this mode makes no claim there)."""
    wl = make_config(3, "full")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    inv = net.graph.inv_perm.long()
    for sched in (0, DATAFLOW):
        _, V, _ = run_gpu(amd, wl, flags=sched | amd.FLAG_ACC_F32, net=net)
        err, any_nan = _max_abs_err_every_element(V, inv, want)
        print(f"config 3 fast mode schedule {sched}: max_abs_err={err:.3e}")
        assert not any_nan and err <= TOL, (sched, err)
        del V


def _per_network(wl, k):
    """Network k of a population workload as a workload of its own (ids and rows made local)."""
    from workloads import Workload
    n0, n1 = int(wl.net_node_ptr[k]), int(wl.net_node_ptr[k + 1])
    e0, e1 = int(wl.net_edge_ptr[k]), int(wl.net_edge_ptr[k + 1])
    i0, i1 = int(wl.net_input_ptr[k]), int(wl.net_input_ptr[k + 1])
    o0, o1 = int(wl.net_output_ptr[k]), int(wl.net_output_ptr[k + 1])
    return Workload(f"{wl.name}[{k}]", n1 - n0, wl.src[e0:e1] - n0, wl.dst[e0:e1] - n0, wl.w[e0:e1],
                    wl.input_ids[i0:i1] - n0, wl.output_ids[o0:o1] - n0, np.ascontiguousarray(wl.X[i0:i1])), (n0, n1, o0, o1)


def test_population_call_equals_per_network_calls(amd):
    """A population is the disjoint union of its networks, so one call over the union must give each
    network what a call of its own gives it.  With level launches and the dataflow schedule the
    order of the additions of a row depends on the row and the batch width alone: bit-identical.
    The workgroup schedule walks the light rows of a narrow level in teams and those of a wide one
    serially (the width of a level differs between the union and one network), so there the two
    agree to the rounding of the final store."""
    wl = make_config(5, "small")
    assert wl.n_nets == 9
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    union = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    lp = union.graph.level_ptr_host
    assert (lp[2::3][: union.n_levels] - lp[1::3][: union.n_levels]).max() < 256    # medium rows are never grouped
    nets = [(_per_network(wl, k)) for k in range(wl.n_nets)]
    singles = [amd.Network(s.n_nodes, s.src, s.dst, s.w, s.input_ids, s.output_ids) for s, _ in nets]
    lv = union.level.cpu().numpy()
    for (s, (n0, n1, _, _)), net in zip(nets, singles):
        assert (net.level.cpu().numpy() == lv[n0:n1]).all()          # levels of the union = per-network levels
    for sched in SCHEDULES:
        _, V, Y = run_gpu(amd, wl, flags=sched, net=union)
        got = union.values_original_order(V).cpu().numpy()
        assert np.abs(got.astype(np.float64) - want).max() <= TIGHT, sched
        y = Y.cpu().numpy()
        for (s, (n0, n1, o0, o1)), net in zip(nets, singles):
            _, Vk, Yk = run_gpu(amd, s, flags=sched, net=net)
            gk = net.values_original_order(Vk).cpu().numpy()
            if sched == WORKGROUP:
                assert np.abs(gk.astype(np.float64) - got[n0:n1]).max() <= TIGHT, (sched, s.name)
                assert np.abs(Yk.cpu().numpy().astype(np.float64) - y[o0:o1]).max() <= TIGHT, (sched, s.name)
            else:
                assert (gk == got[n0:n1]).all(), (sched, s.name)
                assert (Yk.cpu().numpy() == y[o0:o1]).all(), (sched, s.name)


@pytest.mark.parametrize("idx", [3, 4])
def test_relabelled_and_shuffled_network(amd, idx):
    """Renaming the nodes and reordering the connection list changes nothing but names: the levels
    are the same bit for bit, and the activations agree to the rounding of the final store (the
    additions of a row follow the connection list, so the fp64 sums may differ in their last bits)."""
    from workloads import Workload
    wl = make_config(idx, "small")
    rng = np.random.default_rng(77 + idx)
    relabel = rng.permutation(wl.n_nodes).astype(np.int32)           # old id -> new id
    order = rng.permutation(wl.n_edges)
    twin = Workload(wl.name + "-relabelled", wl.n_nodes, relabel[wl.src][order], relabel[wl.dst][order], wl.w[order],
                    relabel[wl.input_ids], relabel[wl.output_ids], wl.X)
    a = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    b = amd.Network(twin.n_nodes, twin.src, twin.dst, twin.w, twin.input_ids, twin.output_ids)
    assert a.n_levels == b.n_levels
    assert (b.level.cpu().numpy()[relabel] == a.level.cpu().numpy()).all()
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        _, Va, Ya = run_gpu(amd, wl, flags=sched, net=a)
        _, Vb, Yb = run_gpu(amd, twin, flags=sched, net=b)
        ga = a.values_original_order(Va).cpu().numpy()
        gb = b.values_original_order(Vb).cpu().numpy()[relabel]
        assert np.abs(ga.astype(np.float64) - gb).max() <= TIGHT, sched
        assert np.abs(gb.astype(np.float64) - want).max() <= TIGHT, sched
        assert np.abs(Ya.cpu().numpy().astype(np.float64) - Yb.cpu().numpy()).max() <= TIGHT, sched


def test_graph_capture_replays_match_eager(amd):
    """asnn_activate enqueues kernels only (no memset, no allocation, no host
    synchronisation), so a stream capture of it replays correctly: several
    replays, with eager work and synchronisations between them, all equal the
    eager result, for every schedule."""
    wl = make_config(3, "small")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    X = torch.from_numpy(wl.X).cuda()
    want_V, want_Y = net.activate(X, flags=LEVELS)
    torch.cuda.synchronize()
    for sched in (LEVELS, DATAFLOW, WORKGROUP):
        V = torch.zeros_like(want_V)
        Y = torch.zeros_like(want_Y)
        net.workspace(wl.B)                       # allocate outside the capture
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            net.activate(X, V=V, Y=Y, flags=sched)           # warm-up on the capture stream
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                net.activate(X, V=V, Y=Y, flags=sched)
        torch.cuda.synchronize()
        for rep in range(3):
            V.fill_(float("nan"))
            Y.fill_(float("nan"))
            X2 = X * 0.5 if rep == 1 else X           # replay reads X in place: change and restore it
            if rep == 1:
                X.copy_(X2)
            graph.replay()
            torch.cuda.synchronize()
            if rep == 1:
                ref_V, ref_Y = net.activate(X2.contiguous(), flags=LEVELS)
                torch.cuda.synchronize()
                assert torch.equal(V, ref_V) and torch.equal(Y, ref_Y)
                X.copy_(torch.from_numpy(wl.X).cuda())
            else:
                assert torch.equal(V, want_V) and torch.equal(Y, want_Y), (sched, rep)
            net.activate(X, flags=sched)              # eager work between replays
            net.check(wl.B)


def test_dataflow_wait_is_bounded_and_reported(amd):
    """Failure handling of the persistent schedule, forced from the host: a
    packed record whose first unit above level 0 is skipped leaves rows that
    nobody writes.  Their consumers must give up after the time limit, every
    wave must still exit, and asnn_activate_status must report the timeout.
    The next, valid activation on the same workspace is clean again."""
    import copy
    import ctypes
    import time
    wl = make_config(3, "small")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    good_V, _ = net.activate(wl.X, flags=DATAFLOW)
    net.check(wl.B)
    g = net.graph
    broken = copy.copy(g)
    rec = type(g.record)()
    ctypes.pointer(rec)[0] = g.record
    rec.first_unit = g.first_unit + 1
    broken.record = rec
    X = torch.from_numpy(wl.X).cuda()
    t0 = time.time()
    amd.asnn_activate(broken, net.input_ids, X, net.output_ids, flags=DATAFLOW, workspace=net.workspace(wl.B))
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_activate_status(net.workspace(wl.B))
    assert e.value.code == -11
    assert time.time() - t0 < 30
    V, _ = net.activate(wl.X, flags=DATAFLOW)
    net.check(wl.B)
    assert torch.equal(V, good_V)


def test_bound_call_and_yardsticks(amd):
    """An activation whose arguments were marshalled once (Network.bind) gives the bits of the general
    call, launch after launch, on inputs changed in place; the bandwidth yardsticks run on the value
    matrix, read only, and leave their sink alone."""
    wl = make_config(3, "small")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    X = torch.from_numpy(wl.X).cuda()
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        want_V, want_Y = net.activate(X, flags=sched)
        net.check(wl.B)
        bound = net.bind(X, flags=sched)
        for rep in range(3):
            bound.V.fill_(float("nan"))
            bound.Y.fill_(float("nan"))
            bound.launch()
            net.check(wl.B)
            assert torch.equal(bound.V, want_V) and torch.equal(bound.Y, want_Y), (sched, rep)
        X.mul_(0.5)                                   # the bound call reads X in place
        bound.launch()
        net.check(wl.B)
        ref_V, ref_Y = net.activate(X, flags=sched)
        net.check(wl.B)
        assert torch.equal(bound.V, ref_V) and torch.equal(bound.Y, ref_Y), sched
        X.copy_(torch.from_numpy(wl.X).cuda())
    V = torch.rand((1000, 256), device="cuda:0")
    keep = V.clone()
    sink = torch.zeros(64, device="cuda:0")
    amd.asnn_device_read(V, sink)
    amd.asnn_device_gather(V, 300, 11, 7, sink)
    amd.asnn_device_gather(V[:10, :64].contiguous(), 5, 3, 1, sink)       # one tile of 64 columns
    W = torch.empty_like(V)
    amd.asnn_device_copy(W, V)
    torch.cuda.synchronize()
    assert torch.equal(V, keep) and torch.equal(W, keep) and float(sink.abs().sum()) == 0.0
    with pytest.raises(amd.AsnnError):
        amd.asnn_device_gather(torch.rand((10, 65), device="cuda:0"), 5, 3, 1, sink)   # rows of whole tiles only
    # the gather that also stores: every element of a stored row is the sum of what its column loaded, all
    # tiles of a row load the same rows, the source stays as it was, and nothing beyond the rows asked for is written
    for cols in (256, 192, 64):
        rows_of = torch.arange(1000, device="cuda:0", dtype=torch.float32)
        S = rows_of[:, None].expand(1000, cols).contiguous()
        out = torch.full((301, cols), -1.0, device="cuda:0")
        amd.asnn_device_gather_store(S, 11, 7, out[:300])
        torch.cuda.synchronize()
        assert torch.equal(S, rows_of[:, None].expand(1000, cols)) and bool((out[300] == -1.0).all())
        got = out[:300]
        assert bool((got == got[:, :1]).all())                      # one sum per row, in every column of every tile
        assert bool((got >= 0).all()) and bool((got <= 11 * 999).all()) and bool((got == got.round()).all())
        assert got[:, 0].unique().numel() > 250                     # different rows gather different sources
        ones = torch.ones((1000, cols), device="cuda:0")
        amd.asnn_device_gather_store(ones, 11, 3, out[:300])
        torch.cuda.synchronize()
        assert bool((out[:300] == 11.0).all())


def test_schedule_choice_is_reported(amd):
    wl = make_config(3, "small")
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    g = net.graph
    assert amd.asnn_activate_schedule(g, wl.B, True, 0) == "dataflow"       # small levels
    assert amd.asnn_activate_schedule(g, wl.B, False, 0) == "levels"        # no workspace
    assert amd.asnn_activate_schedule(g, wl.B, True, LEVELS) == "levels"
    assert amd.asnn_activate_schedule(g, 1 << 20, True, 0) == "levels"      # big levels
    assert amd.asnn_activate_schedule(g, wl.B, False, WORKGROUP) == "workgroup"
    with pytest.raises(amd.AsnnError):
        amd.asnn_activate_schedule(g, wl.B, False, DATAFLOW)
    with pytest.raises(amd.AsnnError):
        amd.asnn_activate_schedule(g, wl.B, True, LEVELS | WORKGROUP)
    tiny = make_config(1, "full")           # a few hundred connections: one workgroup per tile by default
    tnet = amd.Network(tiny.n_nodes, tiny.src, tiny.dst, tiny.w, tiny.input_ids, tiny.output_ids)
    assert amd.asnn_activate_schedule(tnet.graph, 1, True, 0) == "workgroup"
    assert amd.asnn_activate_schedule(tnet.graph, 8, False, 0) == "workgroup"
    assert amd.asnn_activate_schedule(tnet.graph, 4096, False, 0) == "workgroup"    # 64 tiles, a workgroup each
    assert amd.asnn_activate_schedule(tnet.graph, 1 << 20, False, 0) == "levels"    # more tiles than the chip holds workgroups


@pytest.mark.parametrize("idx,scale", [(1, "small"), (3, "small"), (4, "small"), (5, "small"), (3, "full")])
def test_required_set_and_filtered_activation(amd, idx, scale):
    """The set R of the segmentation algorithm on the GPU: bit-exact mask, the
    kept connections are exactly those that end in R in their original order,
    and activating the kept connections gives the same bits on every node of R."""
    wl = make_config(idx, scale)
    dev = "cuda:0"
    src = torch.from_numpy(wl.src).to(dev); dst = torch.from_numpy(wl.dst).to(dev); w = torch.from_numpy(wl.w).to(dev)
    outs = torch.from_numpy(wl.output_ids).to(dev)
    req, n_req = amd.asnn_required_set(wl.n_nodes, src, dst, outs)
    want = oracle.required(wl.n_nodes, wl.src, wl.dst, wl.output_ids)
    assert (req.cpu().numpy().astype(bool) == want).all() and n_req == int(want.sum())
    ks, kd, kw = amd.asnn_filter_required(wl.n_nodes, src, dst, w, req)
    keep = want[wl.dst]
    assert (ks.cpu().numpy() == wl.src[keep]).all() and (kd.cpu().numpy() == wl.dst[keep]).all()
    assert (kw.cpu().numpy() == wl.w[keep]).all()
    full = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    cut = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids, required_only=True)
    assert cut.n_required == int(want.sum()) and cut.src.numel() == int(keep.sum())
    Vf, Yf = full.activate(wl.X); full.check(wl.B)
    Vc, Yc = cut.activate(wl.X); cut.check(wl.B)
    assert torch.equal(Yf, Yc)
    vf = full.values_original_order(Vf).cpu().numpy(); vc = cut.values_original_order(Vc).cpu().numpy()
    assert (vf[want] == vc[want]).all()
    # an output id listed twice, or none at all
    req2, n2 = amd.asnn_required_set(wl.n_nodes, src, dst, torch.cat([outs, outs[:1]]))
    assert n2 == n_req and torch.equal(req2, req)
    req0, n0 = amd.asnn_required_set(wl.n_nodes, src, dst, outs[:0])
    assert n0 == 0 and int(req0.sum()) == 0
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_required_set(wl.n_nodes, src, dst, torch.tensor([wl.n_nodes], dtype=torch.int32, device=dev))
    assert e.value.code == -3


@pytest.mark.parametrize("idx,scale,n_outputs", [(1, "full", 2), (3, "small", 3), (4, "small", 2), (3, "full", 5)])
def test_compacted_required_network(amd, idx, scale, n_outputs):
    """Outputs-only activation: the network restricted to the required set R and renumbered densely.
    The value matrix has |R| rows (nothing outside R is allocated or written), every node of R gets
    the oracle's value of the full network, and Y equals the full network's Y.  Few outputs, so that R
    leaves a good part of the network out; a sensor outside R is skipped."""
    wl = make_config(idx, scale)
    outs = wl.output_ids[:n_outputs]
    want_R = oracle.required(wl.n_nodes, wl.src, wl.dst, outs)
    assert 0 < want_R.sum() < wl.n_nodes
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    full = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, outs)
    cut = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, outs, compact=True)
    n_R = int(want_R.sum())
    assert cut.n_nodes == n_R and cut.n_required == n_R and cut.n_nodes_original == wl.n_nodes
    new_id = cut.new_id.cpu().numpy()
    assert ((new_id >= 0) == want_R).all()
    assert (new_id[want_R] == np.arange(n_R)).all()                   # dense, in the order of the old ids
    assert (cut.input_ids.cpu().numpy() == new_id[wl.input_ids]).all()
    # the compacted network's levels are the full network's levels of the same nodes
    lv, _ = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    assert (cut.level.cpu().numpy() == lv[want_R]).all()
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        V = torch.full((n_R, wl.B), float("nan"), device="cuda:0")
        V, Y = cut.activate(wl.X, V=V, flags=sched)
        cut.check(wl.B)
        assert V.shape == (n_R, wl.B)
        got = cut.values_original_order(V).cpu().numpy()               # indexed by the compacted ids
        err = float(np.abs(got.astype(np.float64) - want[want_R]).max())
        assert err <= TIGHT, (sched, err)
        Vf, Yf = full.activate(wl.X, flags=sched)
        full.check(wl.B)
        assert np.abs(Y.cpu().numpy().astype(np.float64) - Yf.cpu().numpy()).max() <= TIGHT, sched
        assert (Y.cpu().numpy() == got[new_id[outs]]).all(), sched


@pytest.mark.parametrize("idx", [3, 4, 5])
def test_teacher_forced_single_level_error(amd, idx):
    """Every node computed from the ORACLE's values of its sources (one hop), so the error of one
    weighted sum + sigmoid is seen without the amplification along the levels: the end-to-end
    error of the fp32 fast mode on deep networks is amplification of a per-node error of a few
    1e-7, not a kernel defect.  The forced network has 2N nodes: node i carries the oracle's
    value of node i as a raw sensor input, node N+j receives the connections of node j."""
    from workloads import Workload
    wl = make_config(idx, "small")
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)      # float64 holding fp32 values
    n = wl.n_nodes
    has_in = np.bincount(wl.dst, minlength=n) > 0
    forced = Workload("forced", 2 * n, wl.src, (wl.dst + n).astype(np.int32), wl.w, np.arange(n, dtype=np.int32),
                      (np.nonzero(has_in)[0] + n).astype(np.int32), want.astype(np.float32))
    net = None
    for sched in SCHEDULES:
        for fast, bound in ((0, 6.0e-8), (amd.FLAG_ACC_F32, 2.0e-6)):
            net, V, Y = run_gpu(amd, forced, flags=sched | fast | amd.FLAG_RAW_INPUTS, net=net)
            err = float(np.abs(Y.cpu().numpy().astype(np.float64) - want[has_in]).max())
            print(f"config {idx} small, schedule {sched}, fp32 sums {bool(fast)}: single-level max_abs_err {err:.2e}")
            assert err <= bound, (sched, fast, err)


def test_value_matrix_beyond_4_gib(amd):
    """n_nodes * B * 4 >= 4 GiB: every schedule indexes the value matrix with 64 bits (the dataflow
    schedule addresses its tiles through 64-bit global accesses of device scope, not through the
    32-bit offsets of a buffer descriptor).  Parity on sampled batch columns, first, middle and
    last rows written, for the default choice and every forced schedule."""
    wl = layered_skip(seed=5, n_nodes=1_100_000, n_inputs=64, n_outputs=64, n_levels=6, mean_extra_degree=1.0, B=8)
    B = 1024
    assert wl.n_nodes * B * 4 >= 1 << 32
    rng = np.random.default_rng(11)
    X = rng.random((len(wl.input_ids), B), dtype=np.float32)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    assert amd.asnn_activate_schedule(net.graph, B, True, DATAFLOW) == "dataflow"
    cols = np.array([0, 511, 1023])
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, np.ascontiguousarray(X[:, cols]))
    inv = net.graph.inv_perm.long()
    tcols = torch.as_tensor(cols, device="cuda:0")
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        V = torch.full((wl.n_nodes, B), float("nan"), device="cuda:0")
        V, Y = net.activate(X, V=V, flags=sched)
        net.check(B)
        got = V[:, tcols][inv].cpu().numpy()
        err = float(np.abs(got.astype(np.float64) - want).max())
        assert err <= TIGHT, (sched, err)
        assert not torch.isnan(V[-1]).any() and not torch.isnan(V[wl.n_nodes // 2]).any() and not torch.isnan(V[0]).any()
        assert torch.equal(Y, V[inv[net.output_ids.long()]]), sched
        del V, Y


def _random_network(seed):
    """Random DAG with parallel connections, roots that are no sensors, a few very heavy nodes
    (in-degrees around the chunking limits of the dataflow schedule) and several components."""
    from workloads import Workload
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(2, 400))
    order = rng.permutation(n)                         # order[k] = id of the k-th node in topological order
    n_edges = int(rng.integers(0, 6 * n))
    a = rng.integers(0, n - 1, size=n_edges)
    b = rng.integers(0, n, size=n_edges)
    lo, hi = np.minimum(a, b), np.maximum(a, b)
    keep = lo < hi
    src, dst = list(order[lo[keep]]), list(order[hi[keep]])
    for d in rng.choice([40, 255, 256, 300, 511, 512, 513, 1024, 1025, 8192, 8193, 9000], size=int(rng.integers(0, 4))):
        k = int(rng.integers(1, n))                    # position of the heavy node; its sources come before it
        src += list(order[rng.integers(0, k, size=int(d))])
        dst += [order[k]] * int(d)
    src = np.array(src, dtype=np.int32); dst = np.array(dst, dtype=np.int32)
    w = rng.uniform(-1.5, 1.5, size=src.shape[0]).astype(np.float32)
    indeg = np.bincount(dst, minlength=n)
    roots = np.nonzero(indeg == 0)[0]
    inputs = rng.permutation(roots)[: max(1, len(roots) * 2 // 3)].astype(np.int32)      # the other roots stay at 0.5
    outputs = rng.permutation(n)[: int(rng.integers(1, n + 1))].astype(np.int32)
    B = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64, 65, 128, 200, 256, 300]))
    X = rng.uniform(-1, 2, size=(len(inputs), B)).astype(np.float32)
    return Workload(f"random{seed}", n, src, dst, w, inputs, outputs, X)


@pytest.mark.parametrize("seed", range(24))
def test_random_networks_every_schedule_and_mode(amd, seed):
    wl = _random_network(seed)
    lv_o, nl_o = oracle.levels(wl.n_nodes, wl.src, wl.dst)
    want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    assert net.n_levels == nl_o and (net.level.cpu().numpy() == lv_o).all()
    for sched in (0, LEVELS, DATAFLOW, WORKGROUP):
        for fast, bound in ((0, TIGHT), (amd.FLAG_ACC_F32, 30 * TOL)):
            _, V, Y = run_gpu(amd, wl, flags=sched | fast, net=net)
            got = net.values_original_order(V).cpu().numpy()
            err = float(np.abs(got.astype(np.float64) - want).max())
            assert err <= bound, (seed, sched, fast, wl.n_nodes, wl.n_edges, wl.B, err)
            assert (Y.cpu().numpy() == got[wl.output_ids]).all()
