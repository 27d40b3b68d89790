"""Full-size GPU parity, in the launch configuration bench.py times (all K nodes, every tensor of the workload,
fit -> quantize_all -> step, the second round against the first round's messages).

The oracle does about 25 million node-coordinates per second and thread; spread over the box's threads that is enough
to redo whole messages: every tensor of every node, byte for byte, for all three layer-shaped workloads (the DCGAN- and
Transformer-XL-shaped ones for two rounds with every iterate; the 1.3e9-coordinate one for all 16 nodes in round 1,
then two nodes and pieces).  A second test runs the workloads' own round counts with device-side checks every round and
the oracle on pieces of the last one."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2505_14371_amd import qoda, workloads  # noqa: E402

OCT = 2048


def uniform_levels(S):
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


class Full:
    def __init__(self, name):
        if not torch.cuda.is_available():
            pytest.fail("a GPU test was selected but no GPU is visible")
        self.dev = torch.device("cuda:0")
        self.w = w = workloads.get(name)
        self.L, self.K, self.S = len(w.sizes), w.num_nodes, w.points
        self.ctx = qoda.Context(w.sizes, list(range(self.L)), [self.S] * self.L, self.K, w.seed)
        self.off, self.n = workloads.padded_offsets(w.sizes)
        self.grad = [torch.zeros(self.n, dtype=torch.float32, device=self.dev) for _ in range(self.K)]
        self.mbytes = self.ctx.message_bytes()
        self.msg = [[torch.zeros(self.mbytes, dtype=torch.uint8, device=self.dev) for _ in range(self.K)] for _ in range(2)]
        gen = torch.Generator(device=self.dev)
        gen.manual_seed(1234 + w.seed)
        self.x1 = torch.randn(self.n, dtype=torch.float32, device=self.dev, generator=gen)
        self.y = torch.zeros_like(self.x1)
        self.xh = torch.zeros_like(self.x1)
        self.acc = torch.zeros(1, dtype=torch.float64, device=self.dev)
        self.eta = torch.ones(2, dtype=torch.float32, device=self.dev)
        self.hdr_off, self.body_off = self.ctx.message_layout()
        self.c1 = 1 + max(1, int(np.ceil(np.log2(self.S))))

    def ptrs(self, t):
        return [t.data_ptr() + 4 * int(o) for o in self.off]

    def gptrs(self):
        return [p for k in range(self.K) for p in self.ptrs(self.grad[k])]

    def fill(self, round_):
        for k in range(self.K):
            workloads.node_torch(self.w, k, round_, self.dev, out=self.grad[k])

    def layer(self, flat, l, e0=0, e1=None):
        e1 = self.w.sizes[l] if e1 is None else e1
        return flat[int(self.off[l]) + e0: int(self.off[l]) + e1].cpu().numpy()

    def round_(self, t):
        cur = (t - 1) & 1
        if self.w.adaptive:
            self.ctx.fit_levels_keep_norms(self.gptrs(), t)        # as bench.py does: the round's own vectors
        self.ctx.quantize_all(self.gptrs(), t, self.msg[cur], self.msg[1 - cur] if t > 1 else None)
        deltas = self.ctx.read_buffer(qoda.BUF_DELTA)
        acc_before = float(self.acc.cpu()[0])
        self.ctx.step(self.msg[cur], self.ptrs(self.x1), self.ptrs(self.y), self.ptrs(self.xh), self.acc, None, self.eta)
        torch.cuda.synchronize()
        return cur, deltas, acc_before

    def header(self, msg_host, l):
        h = msg_host[int(self.hdr_off[l]): int(self.hdr_off[l]) + 4 * (1 + self.S)].view(np.float32)
        return h[0], h[1:].copy()

    def body_slice(self, msg, l, e0, e1):
        """Packed bytes of the octets covering coordinates [e0, e1) of layer l (e0 a multiple of 2048)."""
        o0, o1 = e0 // OCT, (e1 + OCT - 1) // OCT
        b0 = int(self.body_off[l]) + o0 * 256 * self.c1
        return msg[b0: b0 + (o1 - o0) * 256 * self.c1].cpu().numpy()


def pieces_for(w, whole_limit=3_000_000):
    """(layer, e0, e1): whole tensors when small, else the first octets, a middle run and the ragged tail."""
    L = len(w.sizes)
    big = int(np.argmax(w.sizes))
    layers = sorted({0, 1, 2, 3, min(10, L - 1), big, L - 2, L - 1} & set(range(L)))
    out = []
    for l in layers:
        d = w.sizes[l]
        if d <= whole_limit:
            out.append((l, 0, d))
        else:
            mid = (d // 2) // OCT * OCT
            tail = (d - 1) // OCT * OCT - 2 * OCT
            out += [(l, 0, 3 * OCT), (l, mid, mid + 2 * OCT), (l, tail, d)]
    return out


def _pool(n=None):
    """Threads for the oracle's per-(layer, node) work: its C routines release the interpreter lock.  Sized to the GPU
    box's CPU share."""
    import concurrent.futures
    import os

    return concurrent.futures.ThreadPoolExecutor(max_workers=n or min(16, os.cpu_count() or 1))


def _whole_round(oracle, f, t, prev_levels, prev_msgs, check_iterates):
    """One round in bench.py's configuration, then EVERYTHING against the oracle: per (node, layer) statistic, norm and
    reciprocal; per layer histogram, pooled weights and fitted levels; every node's whole message byte for byte
    (header, every code of every tensor, padding); every node's step-size term recomputed from its stored messages;
    the step size; and (check_iterates) Y and X_{t+3/2} on every coordinate.  Gradients come back from the device
    layer by layer; the oracle's work is spread over threads."""
    w, K, L, S = f.w, f.K, f.L, f.S
    f.fill(t)
    y_old = f.y.clone() if check_iterates else None
    cur, deltas, acc_before = f.round_(t)
    assert f.ctx.status() == qoda.OK
    ss = f.ctx.read_buffer(qoda.BUF_SUMSQ)
    nr = f.ctx.read_buffer(qoda.BUF_NORM)
    iv = f.ctx.read_buffer(qoda.BUF_INV)
    hist = f.ctx.read_buffer(qoda.BUF_HIST) if w.adaptive else None
    pooled = f.ctx.read_buffer(qoda.BUF_POOLED) if w.adaptive else None
    got_levels = [f.ctx.get_levels(l) for l in range(L)]
    msgs = [f.msg[cur][k].cpu().numpy() for k in range(K)]
    hb = int(f.body_off[0])
    want_hdr = oracle.header_bytes(w.sizes, [S] * L)
    assert hb == want_hdr and f.mbytes == oracle.message_bytes(w.sizes, [S] * L)
    levels = [None] * L
    order = sorted(range(L), key=lambda l: -w.sizes[l])           # big tensors first: better balance over the threads

    def node_task(l, k, host, lev):
        s = oracle.sumsq(host)
        assert ss[k, l] == s, (t, k, l)
        n = oracle.sqrt_floor(s)
        assert nr[k, l] == n and iv[k, l] == oracle.rcp_floor(n), (t, k, l)
        mh_norm, mh_lev = f.header(msgs[k][:hb], l)
        assert mh_norm == n and np.array_equal(mh_lev, lev), (t, k, l)
        sign, idx = oracle.quantize_range(host, 0, w.sizes[l], iv[k, l], lev, w.seed, t, k, l)
        want = oracle.pack_layer(sign, idx, S)
        b0 = int(f.body_off[l])
        assert np.array_equal(msgs[k][b0: b0 + want.size], want), (t, k, l)
        return want.size

    with _pool() as pool:
        pending = []
        for l in order:
            host = [f.layer(f.grad[k], l) for k in range(K)]     # D2H of this layer, all nodes
            if w.adaptive:
                levs, oh, op, st = oracle.fit_levels([w.sizes[l]], [0], [S], K, host, [prev_levels[l]])
                assert st == 0
                assert np.array_equal(hist[:, l, :], oh[:, 0, :]), (t, l)
                assert np.array_equal(pooled[l], op[0]), (t, l)
                levels[l] = levs[0]
            else:
                levels[l] = prev_levels[l]
            assert np.array_equal(got_levels[l], levels[l]), (t, l)
            pending += [pool.submit(node_task, l, k, host[k], levels[l]) for k in range(K)]
            while len(pending) > 64:                             # bound the host copies kept alive
                pending.pop(0).result()
            del host
        body = [0] * K
        for fu in pending:
            fu.result()
        # nothing but zeros between the last body byte and the end of the message
        end = int(f.body_off[L - 1]) + ((w.sizes[L - 1] + OCT - 1) // OCT) * 256 * f.c1
        for k in range(K):
            assert not msgs[k][end:].any() and not msgs[k][4 * sum(1 + S for _ in range(L)): hb].any(), k
        del body
        # step-size terms of every node from its stored messages, then the step size
        fut = [pool.submit(oracle.delta_from_messages, w.sizes, [S] * L, msgs[k], None if prev_msgs is None else prev_msgs[k])
               for k in range(K)]
        for k in range(K):
            assert deltas[k] == fut[k].result(), (t, k)
        acc, eta = oracle.step_size(deltas, acc_before)
        assert float(f.acc.cpu()[0]) == acc and float(f.eta.cpu()[0]) == float(eta)
        if check_iterates:                                       # decode + mean + update of every coordinate
            def layer_task(l):
                d = w.sizes[l]
                nb = ((d + OCT - 1) // OCT) * 256 * f.c1
                sub = []
                for kk in range(K):
                    m = np.zeros(oracle.message_bytes([d], [S]), np.uint8)
                    h0 = int(f.hdr_off[l])
                    m[: 4 * (1 + S)] = msgs[kk][h0: h0 + 4 * (1 + S)]
                    o0 = oracle.header_bytes([d], [S])
                    m[o0: o0 + nb] = msgs[kk][int(f.body_off[l]): int(f.body_off[l]) + nb]
                    sub.append(m)
                mean = oracle.dequant_aggregate([d], [S], sub)[0]
                yv = f.layer(y_old, l)
                _, xh = oracle.oda_update(mean, f.layer(f.x1, l), yv, eta, eta, want_next=False)
                assert np.array_equal(f.layer(f.y, l), yv), (t, l)
                assert np.array_equal(f.layer(f.xh, l), xh), (t, l)
            for fu in [pool.submit(layer_task, l) for l in order]:
                fu.result()
    return levels, msgs


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("name", ["dcgan", "txl", "gpt1p3b"])
def test_full_size_whole_messages(oracle, name):
    """Every workload at its full size, two rounds (the second against the first round's messages): every tensor of
    every node, whole messages byte for byte, and every node's step-size term.  Iterates: every coordinate for the two
    smaller workloads; for the 1.3e9-coordinate one a third round checked on pieces (decoding 2e10 node-coordinates a
    second time on the CPU would double the test's time)."""
    f = Full(name)
    levels = {l: uniform_levels(f.S) for l in range(f.L)}
    levels = [levels[l] for l in range(f.L)]
    if name != "gpt1p3b":
        prev = None
        for t in (1, 2):
            levels, prev = _whole_round(oracle, f, t, levels, prev, check_iterates=True)
        return
    prev = None
    for t in (1, 2):
        levels, prev = _whole_round(oracle, f, t, levels, prev, check_iterates=False)
    del prev
    _pieces_round(oracle, f, 3, levels, [0, f.K - 1], pieces_for(f.w))


def _pieces_round(oracle, f, t, prev_levels_list, check_nodes, pieces):
    """A round checked on pieces the oracle can do one by one: whole small tensors, and octet-aligned slices (first,
    middle, ragged tail) of the big ones, for the given nodes; the step-size term of one node from its two stored
    messages; iterates on the pieces."""
    w, K, L, S = f.w, f.K, f.L, f.S
    layers = sorted({p[0] for p in pieces})
    prev_levels = {l: prev_levels_list[l] for l in layers}
    prev_host = {k: f.msg[(t - 2) & 1][k].cpu().numpy() for k in check_nodes[-1:]} if t > 1 else {}
    f.fill(t)
    y_old = {p: f.layer(f.y, p[0], p[1], p[2]) for p in pieces}
    cur, deltas, acc_before = f.round_(t)
    assert f.ctx.status() == qoda.OK
    ss = f.ctx.read_buffer(qoda.BUF_SUMSQ)
    nr = f.ctx.read_buffer(qoda.BUF_NORM)
    iv = f.ctx.read_buffer(qoda.BUF_INV)
    hist = f.ctx.read_buffer(qoda.BUF_HIST) if w.adaptive else None
    pooled = f.ctx.read_buffer(qoda.BUF_POOLED) if w.adaptive else None
    levels = {}
    for l in layers:
        host = [f.layer(f.grad[k], l) for k in range(K)]
        for k in range(K):
            s = oracle.sumsq(host[k])
            assert ss[k, l] == s, (t, k, l)
            n = oracle.sqrt_floor(s)
            assert nr[k, l] == n and iv[k, l] == oracle.rcp_floor(n)
        if w.adaptive:
            levs, oh, op, st = oracle.fit_levels([w.sizes[l]], [0], [S], K, host, [prev_levels[l]])
            assert st == 0
            assert np.array_equal(hist[:, l, :], oh[:, 0, :]), (t, l)
            assert np.array_equal(pooled[l], op[0]), (t, l)
            levels[l] = levs[0]
            assert np.array_equal(f.ctx.get_levels(l), levs[0]), (t, l)
        else:
            levels[l] = prev_levels[l]
        for k in check_nodes:
            mh_norm, mh_lev = f.header(f.msg[cur][k][: int(f.body_off[0])].cpu().numpy(), l)
            assert mh_norm == nr[k, l] and np.array_equal(mh_lev, levels[l])
            for (pl, e0, e1) in pieces:
                if pl != l:
                    continue
                sign, idx = oracle.quantize_range(host[k], e0, e1, iv[k, l], levels[l], w.seed, t, k, l)
                gs, gi = oracle.unpack_layer(f.body_slice(f.msg[cur][k], l, e0, e1), e1 - e0, S)
                assert np.array_equal(gs, sign) and np.array_equal(gi, idx), (t, k, l, e0)
        del host
    k = check_nodes[-1]
    want = oracle.delta_from_messages(w.sizes, [S] * L, f.msg[cur][k].cpu().numpy(), prev_host.get(k))
    assert deltas[k] == want, (t, k)
    acc, eta = oracle.step_size(deltas, acc_before)
    assert float(f.acc.cpu()[0]) == acc and float(f.eta.cpu()[0]) == float(eta)
    for (l, e0, e1) in pieces:
        sub = []
        for kk in range(K):
            hdr = f.msg[cur][kk][int(f.hdr_off[l]): int(f.hdr_off[l]) + 4 * (1 + S)].cpu().numpy()
            body = f.body_slice(f.msg[cur][kk], l, e0, e1)
            hb = oracle.header_bytes([e1 - e0], [S])
            m = np.zeros(oracle.message_bytes([e1 - e0], [S]), np.uint8)
            m[: hdr.size] = hdr
            m[hb: hb + body.size] = body
            sub.append(m)
        mean = oracle.dequant_aggregate([e1 - e0], [S], sub)[0]
        yv = y_old[(l, e0, e1)].copy()
        _, xh = oracle.oda_update(mean, f.layer(f.x1, l, e0, e1), yv, eta, eta, want_next=False)
        assert np.array_equal(f.layer(f.y, l, e0, e1), yv), (t, l, e0)
        assert np.array_equal(f.layer(f.xh, l, e0, e1), xh), (t, l, e0)
    return levels


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("name", ["dcgan", "txl", "gpt1p3b"])
def test_full_size_named_round_counts(oracle, name):
    """The workloads' own round counts at full size (100, 20, 10 rounds; fit every round), so that the state that
    accumulates -- Y, the step-size sum, levels that move, double-buffered messages -- is carried as far as the
    workload says.  Every round is checked on the device with operations that hold bit for bit: Y_{t+1} = Y_t - mean_t
    and X_{t+3/2} = (X_1 + eta Y_{t+1}) - gamma mean_t with the mean from qoda_dequant_aggregate and the same fp32
    operations in torch; eta never grows; the status stays clean.  The last round is checked against the oracle on
    pieces, with the levels fitted by then."""
    f = Full(name)
    w, K, L = f.w, f.K, f.L
    mean = torch.zeros_like(f.x1)
    y_ref = torch.zeros_like(f.x1)
    last_eta = 1.0
    pieces = pieces_for(w, whole_limit=300_000)[:10]
    for t in range(1, w.rounds):
        f.fill(t)
        cur, deltas, _ = f.round_(t)
        f.ctx.dequant_aggregate(f.msg[cur], f.ptrs(mean))
        torch.cuda.synchronize()
        eta = float(f.eta.cpu()[0])
        assert f.ctx.status() == qoda.OK and 0.0 < eta <= last_eta, t
        last_eta = eta
        y_ref -= mean                                            # the kernel's own operation: one fp32 subtraction
        assert torch.equal(f.y, y_ref), t
        want_xh = (f.x1 + f.eta[0] * f.y) - f.eta[1] * mean      # two fp32 operations each, as in the kernel
        for l in range(L):                                       # (the gaps between layers are not state)
            o, d = int(f.off[l]), w.sizes[l]
            assert torch.equal(f.xh[o: o + d], want_xh[o: o + d]), (t, l)
        del want_xh
    lev = [f.ctx.get_levels(l) for l in range(L)]
    _pieces_round(oracle, f, w.rounds, lev, [0, K - 1], pieces)
    assert float(f.eta.cpu()[0]) <= last_eta


@pytest.mark.timeout(900)
def test_full_size_alternative_step_sizes(oracle):
    """eq. (Alt) on the Transformer-XL-shaped workload, two rounds: both rates bit for bit from the sums, lambda
    from one node's norm term recomputed by the oracle from its stored message, mu against a float64 sum over the
    GPU's own fp32 iterates (a property that holds at any size), iterates on the sampled pieces."""
    f = Full("txl")
    w, K, L, S = f.w, f.K, f.L, f.S
    q = 0.25
    sums = torch.zeros(2, dtype=torch.float64, device=f.dev)
    xn = torch.zeros_like(f.x1)
    pieces = pieces_for(w)
    x_prev = f.x1.cpu().numpy().astype(np.float64)          # X_1
    lam = mu = 0.0
    for t in (1, 2):
        f.fill(t)
        cur = (t - 1) & 1
        y_old = {p: f.layer(f.y, p[0], p[1], p[2]) for p in pieces}
        f.ctx.fit_levels(f.gptrs(), t)
        f.ctx.quantize_all(f.gptrs(), t, f.msg[cur], None)
        deltas = f.ctx.read_buffer(qoda.BUF_DELTA)
        eta_prev = float(f.eta.cpu()[0])
        want_eta, want_gamma = oracle.alt_step_size(lam, mu, q)
        f.ctx.step_alt(f.msg[cur], f.ptrs(f.x1), f.ptrs(f.y), f.ptrs(f.xh), sums, f.eta, q, f.ptrs(xn))
        torch.cuda.synchronize()
        assert f.ctx.status() == qoda.OK
        eta = f.eta.cpu().numpy()
        assert eta[0] == want_eta and eta[1] == want_gamma, t
        got = sums.cpu().numpy()
        k = K - 1
        assert deltas[k] == oracle.delta_from_messages(w.sizes, [S] * L, f.msg[cur][k].cpu().numpy(), None)
        lam, _ = oracle.alt_advance(deltas, 0.0, lam, mu)
        assert got[0] == lam
        x_cur = xn.cpu().numpy().astype(np.float64)
        dx2 = sum(float(np.sum((x_prev[int(o): int(o) + d] - x_cur[int(o): int(o) + d]) ** 2))
                  for o, d in zip(f.off, w.sizes))           # layers only: the padding between them is not state
        assert got[1] - mu == pytest.approx(dx2, rel=1e-5), t
        mu = float(got[1])
        x_prev = x_cur
        for (l, e0, e1) in pieces:
            sub = []
            for kk in range(K):
                hdr = f.msg[cur][kk][int(f.hdr_off[l]): int(f.hdr_off[l]) + 4 * (1 + S)].cpu().numpy()
                body = f.body_slice(f.msg[cur][kk], l, e0, e1)
                hb = oracle.header_bytes([e1 - e0], [S])
                m = np.zeros(oracle.message_bytes([e1 - e0], [S]), np.uint8)
                m[: hdr.size] = hdr
                m[hb: hb + body.size] = body
                sub.append(m)
            mean = oracle.dequant_aggregate([e1 - e0], [S], sub)
            yv = [y_old[(l, e0, e1)].copy()]
            x1 = [f.layer(f.x1, l, e0, e1)]
            wxn, wxh, _ = oracle.oda_update_alt([e1 - e0], mean, x1, yv, eta_prev, eta[0], eta[1])
            assert np.array_equal(f.layer(f.y, l, e0, e1), yv[0]), (t, l, e0)
            assert np.array_equal(f.layer(f.xh, l, e0, e1), wxh[0]), (t, l, e0)
            assert np.array_equal(f.layer(xn, l, e0, e1), wxn[0]), (t, l, e0)
    assert mu > 0 and lam > 0


@pytest.mark.timeout(900)
def test_full_size_bucket_scope(oracle):
    """Bucket scope on the Transformer-XL-shaped workload, three rounds in bench.py's configuration (explicit fit in
    round 1, fits from the gathered statistics afterwards): whole small tensors against the oracle (messages with their
    bucket norms, gathered statistics, fitted levels), slices of the big ones, the step-size term of one node
    recomputed from its stored messages, iterates on the pieces."""
    from paper_2505_14371_amd import qoda as q

    name = "txl"
    w = workloads.get(name)
    L, K, S = len(w.sizes), w.num_nodes, w.points
    dev = torch.device("cuda:0")
    ctx = q.Context(w.sizes, list(range(L)), [S] * L, K, w.seed, norm_scope=q.SCOPE_BUCKET)
    off, n = workloads.padded_offsets(w.sizes)
    grad = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(K)]
    mb = ctx.message_bytes()
    msg = [[torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(K)] for _ in range(2)]
    x1 = torch.randn(n, dtype=torch.float32, device=dev)
    y = torch.zeros_like(x1)
    xh = torch.zeros_like(x1)
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, dtype=torch.float32, device=dev)
    ptrs = lambda t: [t.data_ptr() + 4 * int(o) for o in off]
    gp = lambda: [p for k in range(K) for p in ptrs(grad[k])]
    hdr_off, body_off = ctx.message_layout()
    ob = 256 * 4 + 64
    small = [l for l in range(L) if w.sizes[l] <= 200_000][:6] + [L - 1]
    levels = {l: uniform_levels(S) for l in small}
    exps = {}
    stats = {}
    prev_small = {(k, l): None for k in range(K) for l in small}
    for t in (1, 2, 3):
        for k in range(K):
            workloads.node_torch(w, k, t, dev, out=grad[k])
        cur = (t - 1) & 1
        ctx.fit_levels(gp() if t == 1 else None, t)
        host = {(k, l): grad[k][int(off[l]): int(off[l]) + w.sizes[l]].cpu().numpy() for k in range(K) for l in small}
        for l in small:                                      # every layer is its own type: fit layer by layer
            if t == 1:
                lev, _, _, st = oracle.fit_levels([w.sizes[l]], [0], [S], K, [host[(k, l)] for k in range(K)], [levels[l]],
                                                  scope=q.SCOPE_BUCKET)
                b0 = np.stack([oracle.quantize([w.sizes[l]], [S], [lev[0]], [host[(k, l)]], w.seed, 0, k, scope=q.SCOPE_BUCKET,
                                               stats_exp=[oracle.TYPE_SKIP])[5] for k in range(K)])
                _, _, ex, _ = oracle.fit_from_stats([0], [S], K, np.zeros((K, 1, 257), np.uint64), b0, [oracle.TYPE_SKIP], lev)
            else:
                lev, _, ex, st = oracle.fit_from_stats([0], [S], K, stats[l][0], stats[l][1], [exps[l]], [levels[l]])
            levels[l], exps[l] = lev[0], int(ex[0])
            assert np.array_equal(ctx.get_levels(l), levels[l]), (t, l)
        ctx.quantize_all(gp(), t, msg[cur], msg[1 - cur] if t > 1 else None)
        deltas = ctx.read_buffer(q.BUF_DELTA)
        acc_before = float(acc.cpu()[0])
        y_old = y.clone()
        ctx.step(msg[cur], ptrs(x1), ptrs(y), ptrs(xh), acc, None, eta)
        torch.cuda.synchronize()
        assert ctx.status() == q.OK
        for l in small:                                      # whole small tensors: bytes of the body, gathered statistics
            nb = (w.sizes[l] + 2047) // 2048 * ob
            hist = np.zeros((K, 1, 257), np.uint64)
            bmax = np.zeros((K, 1))
            for k in range(K):
                out = oracle.quantize([w.sizes[l]], [S], [levels[l]], [host[(k, l)]], w.seed, t, k,
                                      msg_prev=prev_small[(k, l)], scope=q.SCOPE_BUCKET, stats_exp=[exps[l]])
                # the oracle numbers this tensor as layer 0: draws differ unless the layer index matches, so only
                # layer 0 of the model can be compared byte for byte; for the others compare norms and statistics
                got = msg[cur][k][int(body_off[l]): int(body_off[l]) + nb].cpu().numpy()
                hb = oracle.header_bytes([w.sizes[l]], [S], q.SCOPE_BUCKET)
                _, _, want_norms = oracle.unpack_layer(out[0][hb: hb + nb], w.sizes[l], S, q.SCOPE_BUCKET)
                _, _, got_norms = oracle.unpack_layer(got, w.sizes[l], S, q.SCOPE_BUCKET)
                assert np.array_equal(got_norms, want_norms), (t, k, l)
                hist[k, 0], bmax[k, 0] = out[4][0], out[5][0]
                prev_small[(k, l)] = None                    # (previous messages of other layer numbers are not comparable)
            stats[l] = (hist, bmax)
        # codes of slices, with the right layer number, from the stored bucket norms
        whole = {}
        for (l, e0, e1) in pieces_for(w)[:8]:
            for k in (0, K - 1):
                if (k, l) not in whole:                      # the draws are indexed by the coordinate inside the layer
                    whole = {kk: v for kk, v in whole.items() if kk[1] == l}
                    whole[(k, l)] = grad[k][int(off[l]): int(off[l]) + w.sizes[l]].cpu().numpy()
                g = whole[(k, l)]
                body = msg[cur][k][int(body_off[l]) + e0 // 2048 * ob: int(body_off[l]) + (e1 + 2047) // 2048 * ob].cpu().numpy()
                gs, gi, gn = oracle.unpack_layer(body, e1 - e0, S, q.SCOPE_BUCKET)
                lev = ctx.get_levels(l)
                for b in range(e0, e1, 128):
                    b1 = min(b + 128, e1)
                    nrm = oracle.sqrt_floor(oracle.bucket_sumsq(g[b: b1]))
                    assert gn[(b - e0) // 128] == nrm, (t, k, l, b)
                    sign, idx = oracle.quantize_range(g, b, b1, oracle.rcp_floor(nrm), lev, w.seed, t, k, l)
                    assert np.array_equal(gi[b - e0: b1 - e0], idx) and np.array_equal(gs[b - e0: b1 - e0], sign), (t, k, l, b)
        del whole
        k = K - 1
        if t == 3:
            want = oracle.delta_from_messages(w.sizes, [S] * L, msg[cur][k].cpu().numpy(), msg[1 - cur][k].cpu().numpy(),
                                              scope=q.SCOPE_BUCKET)
            assert deltas[k] == want
        a2, e2 = oracle.step_size(deltas, acc_before)
        assert float(acc.cpu()[0]) == a2 and float(eta.cpu()[0]) == float(e2)
        for (l, e0, e1) in pieces_for(w)[:6]:
            sub = []
            for kk in range(K):
                hdr = msg[cur][kk][int(hdr_off[l]): int(hdr_off[l]) + 4 * (1 + S)].cpu().numpy()
                body = msg[cur][kk][int(body_off[l]) + e0 // 2048 * ob: int(body_off[l]) + (e1 + 2047) // 2048 * ob].cpu().numpy()
                hb = oracle.header_bytes([e1 - e0], [S], q.SCOPE_BUCKET)
                m = np.zeros(oracle.message_bytes([e1 - e0], [S], q.SCOPE_BUCKET), np.uint8)
                m[: hdr.size] = hdr
                m[hb: hb + body.size] = body
                sub.append(m)
            mean = oracle.dequant_aggregate([e1 - e0], [S], sub, scope=q.SCOPE_BUCKET)[0]
            yv = y_old[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy().copy()
            xx = x1[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy()
            _, wxh = oracle.oda_update(mean, xx, yv, e2, e2, want_next=False)
            assert np.array_equal(y[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), yv), (t, l, e0)
            assert np.array_equal(xh[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), wxh), (t, l, e0)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("scope,kind", [(qoda.SCOPE_LAYER, qoda.NORM_L1), (qoda.SCOPE_LAYER, qoda.NORM_LINF),
                                        (qoda.SCOPE_VECTOR, qoda.NORM_L2)])
def test_full_size_other_norms_whole_messages(oracle, scope, kind):
    """The Transformer-XL-shaped workload under L1 / L-infinity normalisation and under one norm per node vector:
    two rounds (the second against the first round's messages) at uniform levels, every node's whole message byte for
    byte and every node's step-size term against the oracle's whole-node routine, the mean on every coordinate of
    round 2."""
    w = workloads.get("txl")
    L, K, S = len(w.sizes), w.num_nodes, w.points
    dev = torch.device("cuda:0")
    ctx = qoda.Context(w.sizes, list(range(L)), [S] * L, K, w.seed, norm_scope=scope, norm_kind=kind)
    off, n = workloads.padded_offsets(w.sizes)
    grad = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(K)]
    mb = ctx.message_bytes()
    assert mb == oracle.message_bytes(w.sizes, [S] * L, scope)
    msg = [[torch.zeros(mb, dtype=torch.uint8, device=dev) for _ in range(K)] for _ in range(2)]
    mean = torch.zeros(n, dtype=torch.float32, device=dev)
    ptrs = lambda t: [t.data_ptr() + 4 * int(o) for o in off]
    lev = [uniform_levels(S)] * L
    prev = [None] * K
    for t in (1, 2):
        for k in range(K):
            workloads.node_torch(w, k, t, dev, out=grad[k])
        cur = (t - 1) & 1
        ctx.quantize_all([p for k in range(K) for p in ptrs(grad[k])], t, msg[cur], msg[1 - cur] if t > 1 else None)
        deltas = ctx.read_buffer(qoda.BUF_DELTA)
        torch.cuda.synchronize()
        assert ctx.status() == qoda.OK
        got = [msg[cur][k].cpu().numpy() for k in range(K)]

        def node_task(k):
            flat = grad[k].cpu().numpy()
            layers = [flat[int(o): int(o) + d] for o, d in zip(off, w.sizes)]
            wm, _, dl, st = oracle.quantize(w.sizes, [S] * L, lev, layers, w.seed, t, k, msg_prev=prev[k], scope=scope,
                                            norm_kind=kind)
            assert st == 0, (t, k)
            assert np.array_equal(got[k], wm), (t, k)
            assert deltas[k] == dl, (t, k)

        with _pool(8) as pool:
            for fu in [pool.submit(node_task, k) for k in range(K)]:
                fu.result()
        prev = got
    ctx.dequant_aggregate(msg[cur], ptrs(mean))
    torch.cuda.synchronize()
    want = oracle.dequant_aggregate(w.sizes, [S] * L, prev, scope=scope)
    host = mean.cpu().numpy()
    for l in range(L):
        assert np.array_equal(host[int(off[l]): int(off[l]) + w.sizes[l]], want[l]), l


@pytest.mark.timeout(900)
def test_layer_beyond_32_bit_indices(oracle):
    """One tensor of 2^32 + 10317 entries (coordinate indices beyond both int32 and uint32; the second tensor's
    body sits beyond 2^31 bytes inside the message), one node, fit -> quantize -> step: the sum of squares, the
    histogram and the fitted levels of the big tensor against the oracle in full, codes and iterates on slices
    around 0, 2^31, 2^32 and the ragged tail, the small tensor in full."""
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    dev = torch.device("cuda:0")
    sizes = [(1 << 32) + 5 * OCT + 77, 5000]
    L, K, S, seed = 2, 1, 16, 77
    ctx = qoda.Context(sizes, [0, 1], [S, S], K, seed)
    off, n = workloads.padded_offsets(sizes)
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    grad = torch.empty(n, dtype=torch.float32, device=dev)
    grad.normal_(generator=gen)
    grad.mul_(3e-3)
    x1 = torch.empty(n, dtype=torch.float32, device=dev)
    x1.normal_(generator=gen)
    y = torch.zeros_like(x1)
    xh = torch.zeros_like(x1)
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, dtype=torch.float32, device=dev)
    mb = ctx.message_bytes()
    hdr_off, body_off = ctx.message_layout()
    assert int(body_off[1]) > (1 << 31)
    msg = torch.zeros(mb, dtype=torch.uint8, device=dev)
    ptrs = lambda t: [t.data_ptr() + 4 * int(o) for o in off]
    ctx.fit_levels(ptrs(grad), 1)
    ctx.quantize_all(ptrs(grad), 1, [msg], None)
    deltas = ctx.read_buffer(qoda.BUF_DELTA)
    ctx.step([msg], ptrs(x1), ptrs(y), ptrs(xh), acc, None, eta)
    torch.cuda.synchronize()
    assert ctx.status() == qoda.OK
    ss = ctx.read_buffer(qoda.BUF_SUMSQ)
    nr = ctx.read_buffer(qoda.BUF_NORM)
    iv = ctx.read_buffer(qoda.BUF_INV)
    hist = ctx.read_buffer(qoda.BUF_HIST)
    acc2, eta2 = oracle.step_size(deltas, 0.0)
    assert float(acc.cpu()[0]) == acc2 and float(eta.cpu()[0]) == float(eta2)
    c1 = 5
    d0 = sizes[0]
    tail = (d0 - 1) // OCT * OCT - 2 * OCT
    pieces = {0: [(0, 3 * OCT), ((1 << 31) - 2 * OCT, (1 << 31) + 2 * OCT), ((1 << 32) - 2 * OCT, (1 << 32) + 2 * OCT), (tail, d0)],
              1: [(0, sizes[1])]}
    for l in (0, 1):
        host = grad[int(off[l]): int(off[l]) + sizes[l]].cpu().numpy()
        s = oracle.sumsq(host)
        assert ss[0, l] == s, l
        assert nr[0, l] == oracle.sqrt_floor(s) and iv[0, l] == oracle.rcp_floor(nr[0, l])
        levs, oh, _, st = oracle.fit_levels([sizes[l]], [0], [S], 1, [host], [uniform_levels(S)])
        assert st == 0
        assert np.array_equal(hist[0, l], oh[0, 0]), l
        lev = ctx.get_levels(l)
        assert np.array_equal(lev, levs[0]), l
        for (e0, e1) in pieces[l]:
            b0 = int(body_off[l]) + e0 // OCT * 256 * c1
            body = msg[b0: b0 + (e1 - e0 + OCT - 1) // OCT * 256 * c1].cpu().numpy()
            sign, idx = oracle.quantize_range(host, e0, e1, iv[0, l], lev, seed, 1, 0, l)
            gs, gi = oracle.unpack_layer(body, e1 - e0, S)
            assert np.array_equal(gs, sign) and np.array_equal(gi, idx), (l, e0)
            hdr = msg[int(hdr_off[l]): int(hdr_off[l]) + 4 * (1 + S)].cpu().numpy()
            hb = oracle.header_bytes([e1 - e0], [S])
            m = np.zeros(oracle.message_bytes([e1 - e0], [S]), np.uint8)
            m[: hdr.size] = hdr
            m[hb: hb + body.size] = body
            mean = oracle.dequant_aggregate([e1 - e0], [S], [m])[0]
            yv = np.zeros(e1 - e0, np.float32)
            xx = x1[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy()
            _, wxh = oracle.oda_update(mean, xx, yv, eta2, eta2, want_next=False)
            assert np.array_equal(y[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), yv), (l, e0)
            assert np.array_equal(xh[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), wxh), (l, e0)
        del host
    # the step-size term of the whole message (first round: the previous vectors are zero) against a float64 sum of the
    # decoded values, a property that holds at any size: Y = -mean = -Vhat after one round from Y = 0.  The term is
    # accumulated in fp32 inside each lane's 64 coordinates of a tile (rounding 2^-24 per operation), in fp64 above.
    got = float(torch.sum(y.double() ** 2))
    assert deltas[0] == pytest.approx(got, rel=2e-6)


@pytest.mark.timeout(900)
def test_layer_beyond_32_bit_indices_bucket_scope(oracle):
    """The same oversized tensor under bucket scope (octets of 256*(1+b)+64 bytes: byte offsets beyond 2^32 inside
    the message): fitted levels against the oracle in full; bucket norms, codes and iterates on the slices."""
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    dev = torch.device("cuda:0")
    sizes = [(1 << 32) + 5 * OCT + 77, 5000]
    K, S, seed = 1, 16, 78
    B = qoda.SCOPE_BUCKET
    ctx = qoda.Context(sizes, [0, 1], [S, S], K, seed, norm_scope=B)
    off, n = workloads.padded_offsets(sizes)
    gen = torch.Generator(device=dev)
    gen.manual_seed(100)
    grad = torch.empty(n, dtype=torch.float32, device=dev)
    grad.normal_(generator=gen)
    grad.mul_(3e-3)
    x1 = torch.empty(n, dtype=torch.float32, device=dev)
    x1.normal_(generator=gen)
    y = torch.zeros_like(x1)
    xh = torch.zeros_like(x1)
    acc = torch.zeros(1, dtype=torch.float64, device=dev)
    eta = torch.ones(2, dtype=torch.float32, device=dev)
    mb = ctx.message_bytes()
    hdr_off, body_off = ctx.message_layout()
    assert int(body_off[1]) > (1 << 31)
    msg = torch.zeros(mb, dtype=torch.uint8, device=dev)
    ptrs = lambda t: [t.data_ptr() + 4 * int(o) for o in off]
    ctx.fit_levels(ptrs(grad), 1)
    ctx.quantize_all(ptrs(grad), 1, [msg], None)
    deltas = ctx.read_buffer(qoda.BUF_DELTA)
    ctx.step([msg], ptrs(x1), ptrs(y), ptrs(xh), acc, None, eta)
    torch.cuda.synchronize()
    assert ctx.status() == qoda.OK
    acc2, eta2 = oracle.step_size(deltas, 0.0)
    assert float(acc.cpu()[0]) == acc2 and float(eta.cpu()[0]) == float(eta2)
    ob = 256 * 5 + 64
    d0 = sizes[0]
    tail = (d0 - 1) // OCT * OCT - 2 * OCT
    pieces = {0: [(0, 3 * OCT), ((1 << 31) - 2 * OCT, (1 << 31) + 2 * OCT), ((1 << 32) - 2 * OCT, (1 << 32) + 2 * OCT), (tail, d0)],
              1: [(0, sizes[1])]}
    for l in (0, 1):
        host = grad[int(off[l]): int(off[l]) + sizes[l]].cpu().numpy()
        levs, _, _, st = oracle.fit_levels([sizes[l]], [0], [S], 1, [host], [uniform_levels(S)], scope=B)
        assert st == 0
        lev = ctx.get_levels(l)
        assert np.array_equal(lev, levs[0]), l
        for (e0, e1) in pieces[l]:
            b0 = int(body_off[l]) + e0 // OCT * ob
            body = msg[b0: b0 + (e1 - e0 + OCT - 1) // OCT * ob].cpu().numpy()
            gs, gi, gn = oracle.unpack_layer(body, e1 - e0, S, B)
            for b in range(e0, e1, 128):
                b1 = min(b + 128, e1)
                nrm = oracle.sqrt_floor(oracle.bucket_sumsq(host[b: b1]))
                assert gn[(b - e0) // 128] == nrm, (l, b)
                sign, idx = oracle.quantize_range(host, b, b1, oracle.rcp_floor(nrm), lev, seed, 1, 0, l)
                assert np.array_equal(gi[b - e0: b1 - e0], idx) and np.array_equal(gs[b - e0: b1 - e0], sign), (l, b)
            hdr = msg[int(hdr_off[l]): int(hdr_off[l]) + 4 * (1 + S)].cpu().numpy()
            hb = oracle.header_bytes([e1 - e0], [S], B)
            m = np.zeros(oracle.message_bytes([e1 - e0], [S], B), np.uint8)
            m[: hdr.size] = hdr
            m[hb: hb + body.size] = body
            mean = oracle.dequant_aggregate([e1 - e0], [S], [m], scope=B)[0]
            yv = np.zeros(e1 - e0, np.float32)
            xx = x1[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy()
            _, wxh = oracle.oda_update(mean, xx, yv, eta2, eta2, want_next=False)
            assert np.array_equal(y[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), yv), (l, e0)
            assert np.array_equal(xh[int(off[l]) + e0: int(off[l]) + e1].cpu().numpy(), wxh), (l, e0)
        del host
    got = float(torch.sum(y.double() ** 2))
    assert deltas[0] == pytest.approx(got, rel=2e-6)
