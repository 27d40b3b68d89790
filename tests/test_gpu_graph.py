"""A steady-state round enqueues kernels only, so it can be captured into a HIP graph: two rounds (both message
buffers of the ping-pong) are captured once and replayed several times, with eager work and synchronisations between
the replays; every replay must leave exactly what the same calls leave when issued eagerly."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2505_14371_amd import qoda, workloads  # noqa: E402


@pytest.mark.parametrize("scope", [qoda.SCOPE_LAYER, qoda.SCOPE_BUCKET])
def test_two_rounds_replayed_from_a_graph(scope):
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    dev = torch.device("cuda:0")
    w = workloads.mini("dcgan", max_layer=300000, max_layers=10)
    L, K, S = len(w.sizes), 4, w.points
    ctx = qoda.Context(w.sizes, list(range(L)), [S] * L, K, w.seed, norm_scope=scope)
    off, n = workloads.padded_offsets(w.sizes)
    grad = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(K)]
    ptrs = lambda t: [t.data_ptr() + 4 * int(o) for o in off]
    gp = [p for k in range(K) for p in ptrs(grad[k])]
    mb = ctx.message_bytes()
    msg = [[torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(K)] for _ in range(2)]
    x1 = torch.randn(n, device=dev)
    y = torch.zeros(n, device=dev)
    xh = torch.zeros(n, device=dev)
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, device=dev)
    bucket = scope == qoda.SCOPE_BUCKET

    def fill(r):
        for k in range(K):
            workloads.node_torch(w, k, r, dev, out=grad[k])

    def two_rounds(stream):
        for cur, t in ((0, 2), (1, 3)):
            if bucket:
                ctx.fit_levels(None, t, stream=stream)
            else:
                ctx.fit_levels_keep_norms(gp, t, stream=stream)
            ctx.quantize_all(gp, t, msg[cur], msg[1 - cur], stream=stream)
            ctx.step(msg[cur], ptrs(x1), ptrs(y), ptrs(xh), acc, None, eta, stream=stream)

    def reset():
        y.zero_()
        acc.zero_()
        for k in range(K):
            msg[0][k].zero_()
            msg[1][k].zero_()
        for m in range(L):
            ctx.set_levels(m, (np.arange(S) / (S - 1)).astype(np.float32), stream=s.cuda_stream)
        if bucket:                                   # the same starting scale for both runs
            fill(1)
            ctx.fit_levels(gp, 1, stream=s.cuda_stream)
        torch.cuda.synchronize()

    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        fill(1)
        if bucket:
            ctx.fit_levels(gp, 1, stream=s.cuda_stream)
        two_rounds(s.cuda_stream)                    # first use of every pointer set uploads its table
        torch.cuda.synchronize()
        reset()
        want = []
        for rep in range(3):
            fill(10 + rep)
            two_rounds(s.cuda_stream)
            torch.cuda.synchronize()
            want.append((y.clone(), xh.clone(), acc.clone(), msg[0][1].clone(), msg[1][K - 1].clone(),
                         [ctx.get_levels(m, stream=s.cuda_stream) for m in (0, L - 1)]))
        reset()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        fill(10)
        with torch.cuda.graph(g, stream=s):
            two_rounds(s.cuda_stream)
        reset()                                      # capturing runs nothing; start from the same state
        torch.cuda.synchronize()
        for rep in range(3):
            fill(10 + rep)                           # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = (y, xh, acc, msg[0][1], msg[1][K - 1])
            for a, b in zip(got, want[rep][:5]):
                assert torch.equal(a, b), rep
            for m, lv in zip((0, L - 1), want[rep][5]):
                assert np.array_equal(ctx.get_levels(m, stream=s.cuda_stream), lv), (rep, m)
    assert ctx.status() == qoda.OK
