"""asnn_activate_static: the entry point that allocates nothing.

It must give what asnn_activate gives (same kernels, the library's own scratch in the place of
the caller's workspace), on two calls in a row of which the second is smaller: the scratch still
holds the first call's control block and partial sums when the second starts.  Runs last in the
suite (and must also pass alone in a fresh process).
"""
import numpy as np
import pytest

from workloads import Workload, make_config

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

DATAFLOW = 8


@pytest.fixture(scope="module")
def amd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2005_04347_amd as amd
    amd.load()
    return amd


def _split_rows_network(seed, n_in, n_mid, degrees, B):
    """Two levels above the sensors; the rows of the first have the given in-degrees (those beyond
    512 connections are cut into chunks whose partial sums pass through the scratch), the rows of
    the second gather from everything below."""
    rng = np.random.default_rng(seed)
    n = n_in + n_mid + 4
    src, dst = [], []
    for m in range(n_mid):
        d = degrees[m % len(degrees)]
        src += rng.integers(0, n_in, size=d).tolist()
        dst += [n_in + m] * d
    for t in range(4):
        d = [5, 40, 700, 3000][t]
        src += rng.integers(0, n_in + n_mid, size=d).tolist()
        dst += [n_in + n_mid + t] * d
    src = np.array(src, dtype=np.int32)
    dst = np.array(dst, dtype=np.int32)
    w = rng.uniform(-1, 1, size=src.shape[0]).astype(np.float32)
    X = rng.uniform(0, 1, size=(n_in, B)).astype(np.float32)
    relabel = rng.permutation(n).astype(np.int32)
    order = rng.permutation(src.shape[0])
    return Workload(f"split{seed}", n, relabel[src][order], relabel[dst][order], w[order],
                    relabel[np.arange(n_in)], relabel[np.arange(n - 4, n)], X)


def _both_ways(amd, wl, flags):
    """-> (V, Y) by asnn_activate with a workspace, (V, Y) by asnn_activate_static; all on NaN-poisoned buffers."""
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    B = wl.B
    X = torch.from_numpy(wl.X).cuda()
    nan = float("nan")
    V1 = torch.full((wl.n_nodes, B), nan, device="cuda:0")
    Y1 = torch.full((len(wl.output_ids), B), nan, device="cuda:0")
    amd.asnn_activate(net.graph, net.input_ids, X, net.output_ids, V=V1, Y=Y1, flags=flags, workspace=net.workspace(B))
    net.check(B)
    V2 = torch.full((wl.n_nodes, B), nan, device="cuda:0")
    Y2 = torch.full((len(wl.output_ids), B), nan, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    amd.asnn_activate_static(net.graph, net.input_ids, X, V2, net.output_ids, Y2, flags=flags)
    amd.asnn_activate_status(amd.STATIC_SCRATCH)           # synchronises; raises if a wait gave up
    assert torch.cuda.memory_allocated() == before          # (the binding brought no tensor of its own either)
    return net, (V1, Y1), (V2, Y2)


def test_static_scratch_matches_workspace_on_two_calls_in_a_row(amd):
    import oracle
    # first call: rows of up to 20000 connections at 64 columns (16 chunks, 2 MB of partial sums)
    big = _split_rows_network(1, n_in=400, n_mid=90, degrees=[3, 31, 33, 300, 513, 900, 4096, 20000], B=64)
    # second call, smaller in every respect: fewer rows, fewer chunks, fewer columns (ragged tile)
    small = _split_rows_network(2, n_in=100, n_mid=20, degrees=[2, 40, 600, 1500], B=5)
    for wl in (big, small):
        for flags in (DATAFLOW, 0):
            net, (V1, Y1), (V2, Y2) = _both_ways(amd, wl, flags)
            assert net.graph.record.max_heavy_indegree > 512
            assert not torch.isnan(V2).any() and not torch.isnan(Y2).any()
            assert torch.equal(V1, V2) and torch.equal(Y1, Y2), (wl.name, flags)
            want = oracle.activate(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.X)
            got = net.values_original_order(V2).cpu().numpy()
            assert np.abs(got.astype(np.float64) - want).max() <= 2.5e-7, (wl.name, flags)
    # and once more on an ordinary network, every schedule
    wl = make_config(3, "small")
    for flags in (0, 4, 8, 16):
        _, (V1, Y1), (V2, Y2) = _both_ways(amd, wl, flags)
        assert torch.equal(V1, V2) and torch.equal(Y1, Y2), flags


def test_static_scratch_refuses_what_does_not_fit(amd):
    """A network with split rows at a batch width whose partial sums exceed the scratch is refused
    before anything is launched; the same network at a narrower batch runs."""
    import ctypes
    wl = _split_rows_network(3, n_in=300, n_mid=40, degrees=[10, 700, 5000], B=4)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    lib = amd.load()
    B = 4
    while lib.asnn_activate_workspace_bytes(ctypes.byref(net.graph.record), B) <= amd.STATIC_SCRATCH_BYTES:
        B *= 2
    X = torch.zeros((len(wl.input_ids), B), device="cuda:0")
    V = torch.full((wl.n_nodes, B), float("nan"), device="cuda:0")
    Y = torch.full((len(wl.output_ids), B), float("nan"), device="cuda:0")
    with pytest.raises(amd.AsnnError) as e:
        amd.asnn_activate_static(net.graph, net.input_ids, X, V, net.output_ids, Y)
    assert e.value.code == -12
    torch.cuda.synchronize()
    assert torch.isnan(V).all() and torch.isnan(Y).all()          # nothing ran
    # (a batch that fits runs: covered by the test above)


def test_static_scratch_under_graph_capture(amd):
    """The callers the entry point is for: asnn_activate_static captured in a HIP graph (it enqueues
    kernels only), replayed several times with eager work between the replays, every replay equal to
    the eager result; the dataflow schedule with split rows, whose scratch is the library's own."""
    wl = _split_rows_network(5, n_in=200, n_mid=30, degrees=[4, 50, 700, 2500], B=16)
    net = amd.Network(wl.n_nodes, wl.src, wl.dst, wl.w, wl.input_ids, wl.output_ids)
    X = torch.from_numpy(wl.X).cuda()
    want_V, want_Y = net.activate(X, flags=DATAFLOW)
    net.check(wl.B)
    V = torch.zeros_like(want_V)
    Y = torch.zeros_like(want_Y)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        amd.asnn_activate_static(net.graph, net.input_ids, X, V, net.output_ids, Y, flags=DATAFLOW)      # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            amd.asnn_activate_static(net.graph, net.input_ids, X, V, net.output_ids, Y, flags=DATAFLOW)
    torch.cuda.synchronize()
    for rep in range(3):
        V.fill_(float("nan"))
        Y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(V, want_V) and torch.equal(Y, want_Y), rep
        other = _split_rows_network(6 + rep, n_in=50, n_mid=10, degrees=[3, 600], B=3)       # eager work on the same scratch between replays
        onet = amd.Network(other.n_nodes, other.src, other.dst, other.w, other.input_ids, other.output_ids)
        oV = torch.empty((other.n_nodes, 3), device="cuda:0")
        oY = torch.empty((len(other.output_ids), 3), device="cuda:0")
        amd.asnn_activate_static(onet.graph, onet.input_ids, torch.from_numpy(other.X).cuda(), oV, onet.output_ids, oY, flags=DATAFLOW)
        amd.asnn_activate_status(amd.STATIC_SCRATCH)
