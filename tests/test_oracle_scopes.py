"""Pins for the oracle's other norm scopes: one norm for the node's whole dual vector (the literal reading of
Sec. 2.2 / Sec. 3.1, which normalise "the vector") and one norm per bucket of 128 consecutive entries (the setting
of the experiments, Sec. 7).  What is pinned: the bucket sum against exact arithmetic, the stored norms against
numpy, unbiasedness and the exact variance eq. (Var) with per-bucket norms, on-grid reproduction, independence of
buckets, the cases that reduce to the per-layer scope, message sizes, and the fit's pooled weights recomputed
from the definition."""
import numpy as np
import pytest

from paper_2505_14371_amd import workloads

LAYER, VECTOR, BUCKET = 0, 1, 2


def uniform_levels(S):
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


def test_bucket_sum_of_squares(oracle):
    """Lane sums are fp32 fused chains over 4 coordinates, widened and combined by the in-order binary tree in fp64;
    a result below 2^-100 or not finite is redone with exact fp64 squares."""
    rng = np.random.default_rng(0)
    ints = rng.integers(-2000, 2000, 128).astype(np.float32)           # squares and lane sums below 2^24: all exact
    assert oracle.bucket_sumsq(ints) == float(np.sum(ints.astype(np.int64) ** 2))
    for n in (1, 3, 4, 5, 31, 64, 127, 128):
        v = (rng.standard_t(3, n) * 10.0 ** rng.uniform(-12, 12)).astype(np.float32)
        want = float(np.sum(v.astype(np.float64) ** 2))
        assert oracle.bucket_sumsq(v) == pytest.approx(want, rel=3e-7)  # single precision inside a lane
        padded = np.concatenate([v, np.zeros(128 - n, np.float32)])
        assert oracle.bucket_sumsq(padded) == oracle.bucket_sumsq(v)   # missing coordinates count as zeros
    assert oracle.bucket_sumsq(np.array([4097.0], np.float32)) == 16785408.0   # 4097^2 = 2^24 + 8193 rounded in fp32
    # squares outside the fp32 range: the bucket is redone with exact fp64 squares (same lanes, same tree)
    tiny = np.full(128, 1e-30, np.float32)
    assert oracle.bucket_sumsq(tiny) == pytest.approx(128 * float(tiny[0]) ** 2, rel=1e-15)
    assert oracle.bucket_sumsq(np.array([3e19], np.float32)) == float(np.float32(3e19)) ** 2
    assert oracle.bucket_sumsq(np.array([2.0 ** -149], np.float32)) == 2.0 ** -298
    assert oracle.bucket_sumsq(np.array([np.inf, 1.0], np.float32)) == np.inf and np.isnan(oracle.bucket_sumsq(np.array([np.nan], np.float32)))
    edge = np.zeros(128, np.float32)
    edge[5] = 2.0 ** -50                                               # exactly 2^-100: single precision is kept
    assert oracle.bucket_sumsq(edge) == 2.0 ** -100
    # the combination order is the in-order binary tree in fp64: a case where another order rounds differently
    v = np.zeros(128, np.float32)
    v[0], v[4], v[8], v[12] = 2.0 ** 27, 1.0, 1.0, 2.0 ** 27           # lane sums 2^54, 1, 1, 2^54
    assert oracle.bucket_sumsq(v) == 2.0 ** 55                         # (2^54 + 1) + (1 + 2^54): both round to 2^54
    v[4], v[8] = 2.0 ** 0.5 * 2.0 ** 13, 0.0                           # lane 1: about 2^27, kept by the fp64 tree
    assert oracle.bucket_sumsq(v) == 2.0 ** 55 + float(np.float32(v[4]) * np.float32(v[4]))
    # a lane's own chain: ((2^54 + 1) + 1) + 2^52 in fp32 loses each +1
    w = np.zeros(128, np.float32)
    w[0], w[1], w[2], w[3] = 2.0 ** 27, 1.0, 1.0, 2.0 ** 26
    assert oracle.bucket_sumsq(w) == 2.0 ** 54 + 2.0 ** 52


def _decode_layers(oracle, sizes, S, msg, scope):
    return oracle.dequant_aggregate(sizes, [S] * len(sizes), [msg], scope=scope)


def test_bucket_norms_codes_and_sizes(oracle):
    S, sizes = 8, [1, 127, 128, 129, 2048, 2049, 5000, 0, 40000]
    L = len(sizes)
    lev = [uniform_levels(S)] * L
    rng = np.random.default_rng(1)
    g = [(rng.standard_t(3, s) * 10.0 ** rng.uniform(-4, 2)).astype(np.float32) for s in sizes]
    msg, _, delta, st = oracle.quantize(sizes, [S] * L, lev, g, 7, 1, 0, scope=BUCKET)
    assert st == 0
    hb = oracle.header_bytes(sizes, [S] * L, BUCKET)
    assert hb == oracle.header_bytes(sizes, [S] * L, LAYER)
    extra = sum((s + 2047) // 2048 * 64 for s in sizes)
    want_bytes = hb + sum((s + 2047) // 2048 * 256 * 4 for s in sizes) + extra
    assert msg.size == (want_bytes + 255) // 256 * 256
    _, body = oracle.layout(sizes, [S] * L, BUCKET)
    dec = _decode_layers(oracle, sizes, S, msg, BUCKET)
    total = 0.0
    for l, s in enumerate(sizes):
        if s == 0:
            continue
        nb = (s + 2047) // 2048 * oracle.octet_bytes(S, BUCKET)
        sign, idx, norms = oracle.unpack_layer(msg[int(body[l]): int(body[l]) + nb], s, S, BUCKET)
        assert norms.size == (s + 127) // 128
        for b in range(norms.size):
            seg = g[l][128 * b: 128 * (b + 1)].astype(np.float64)
            true = np.sqrt(np.sum(seg ** 2))
            assert abs(float(norms[b]) - true) <= true * 3e-7          # fp32 lane sums, then the floor of the root
            # each coordinate decodes to +-norm_b * level and lies within one gap of the input
            out = dec[l][128 * b: 128 * (b + 1)]
            want = np.where(sign[128 * b: 128 * (b + 1)] == 1, -1.0, 1.0) * (
                norms[b] * lev[l][idx[128 * b: 128 * (b + 1)]]).astype(np.float32)
            assert np.array_equal(out, want.astype(np.float32))
            assert np.all(np.abs(out.astype(np.float64) - seg) <= float(norms[b]) / (S - 1) * (1 + 1e-6))
        assert np.array_equal(sign, (g[l].view(np.uint32) >> 31).astype(np.uint8))
        total += float(np.sum(dec[l].astype(np.float64) ** 2))
    assert delta == pytest.approx(total, rel=1e-5)                     # no previous message: ||Vhat||^2
    assert oracle.delta_from_messages(sizes, [S] * L, msg, None, scope=BUCKET) == delta


def test_buckets_are_independent_and_layer_scope_is_not(oracle):
    S, d = 16, 1024
    lev = [uniform_levels(S)]
    rng = np.random.default_rng(2)
    a = rng.standard_normal(d).astype(np.float32)
    b = a.copy()
    b[128 * 3 + 5] = 50.0                                              # one entry of bucket 3 becomes large
    ma, _, _, _ = oracle.quantize([d], [S], lev, [a], 3, 1, 0, scope=BUCKET)
    mb, _, _, _ = oracle.quantize([d], [S], lev, [b], 3, 1, 0, scope=BUCKET)
    nb = oracle.octet_bytes(S, BUCKET)
    hb = oracle.header_bytes([d], [S], BUCKET)
    sa, ia, na = oracle.unpack_layer(ma[hb: hb + nb], d, S, BUCKET)
    sb, ib, nbk = oracle.unpack_layer(mb[hb: hb + nb], d, S, BUCKET)
    other = np.ones(d, bool)
    other[128 * 3: 128 * 4] = False
    assert np.array_equal(ia[other], ib[other]) and np.array_equal(np.delete(na, 3), np.delete(nbk, 3))
    assert nbk[3] > 40 and not np.array_equal(ia[~other], ib[~other])
    la, _, _, _ = oracle.quantize([d], [S], lev, [a], 3, 1, 0, scope=LAYER)
    lb, _, _, _ = oracle.quantize([d], [S], lev, [b], 3, 1, 0, scope=LAYER)
    _, il_a = oracle.unpack_layer(la[hb:], d, S)
    _, il_b = oracle.unpack_layer(lb[hb:], d, S)
    assert np.mean(il_a[other] != il_b[other]) > 0.1                   # one norm for the layer: other buckets move too


def test_scopes_coincide_where_they_must(oracle):
    S = 8
    lev = uniform_levels(S)
    ints = np.random.default_rng(3).integers(-100, 100, 128).astype(np.float32)   # all three sums are exact
    ml, sl, dl, _ = oracle.quantize([128], [S], [lev], [ints], 5, 2, 1, scope=LAYER)
    mv, sv, dv, _ = oracle.quantize([128], [S], [lev], [ints], 5, 2, 1, scope=VECTOR)
    mb, _, db, _ = oracle.quantize([128], [S], [lev], [ints], 5, 2, 1, scope=BUCKET)
    assert np.array_equal(ml, mv) and sl[0] == sv[0] and dl == dv                 # one layer: vector = layer
    hb = oracle.header_bytes([128], [S])
    sgl, il = oracle.unpack_layer(ml[hb:], 128, S)
    sgb, ib, nb = oracle.unpack_layer(mb[hb:], 128, S, BUCKET)
    assert np.array_equal(il, ib) and np.array_equal(sgl, sgb)                    # one bucket: same norm, same codes
    assert nb[0] == ml[:4].view(np.float32)[0] and db == dl


def test_vector_scope_uses_one_norm_for_every_layer(oracle):
    S, sizes = 16, [300, 70000, 5, 0, 20000]
    L = len(sizes)
    lev = [uniform_levels(S)] * L
    rng = np.random.default_rng(4)
    g = [(rng.standard_normal(s) * 10.0 ** (l - 2)).astype(np.float32) for l, s in enumerate(sizes)]
    msg, ss, delta, st = oracle.quantize(sizes, [S] * L, lev, g, 11, 1, 2, scope=VECTOR)
    total = sum(float(np.sum(a.astype(np.float64) ** 2)) for a in g)
    assert st == 0 and all(s == ss[0] for s in ss) and ss[0] == pytest.approx(total, rel=1e-14)
    hdr, _ = oracle.layout(sizes, [S] * L, VECTOR)
    norms = [msg[int(h): int(h) + 4].view(np.float32)[0] for h in hdr]
    assert all(n == norms[0] for n in norms) and norms[0] == oracle.sqrt_floor(ss[0])
    assert msg.size == oracle.message_bytes(sizes, [S] * L, LAYER)
    dec = _decode_layers(oracle, sizes, S, msg, VECTOR)
    for l in range(L):
        assert np.all(np.abs(dec[l].astype(np.float64) - g[l]) <= float(norms[0]) / (S - 1) * (1 + 1e-6))
    # the small layers drown under the whole vector's norm: most of their entries fall into the first gap
    assert np.mean(np.abs(dec[0]) == 0) > 0.9


@pytest.mark.parametrize("scope", [VECTOR, BUCKET])
def test_unbiased_with_the_exact_variance(oracle, scope):
    """E[Q(v)] = v and E||Q(v) - v||^2 = sum over norm groups of norm^2 sum_i (l_{tau+1} - u_i)(u_i - l_tau)  (eq. (Var))."""
    S, sizes, seeds = 4, [384, 200], 1500
    L = len(sizes)
    lev = np.array([0.0, 0.2, 0.55, 1.0], np.float32)
    rng = np.random.default_rng(5)
    g = [rng.standard_normal(s).astype(np.float32) * (1 + 3 * l) for l, s in enumerate(sizes)]
    mean = [np.zeros(s) for s in sizes]
    err2 = 0.0
    for seed in range(seeds):
        msg, _, _, _ = oracle.quantize(sizes, [S] * L, [lev] * L, g, seed, 1, 0, scope=scope)
        dec = _decode_layers(oracle, sizes, S, msg, scope)
        for l in range(L):
            mean[l] += dec[l]
            err2 += float(np.sum((dec[l].astype(np.float64) - g[l]) ** 2))
    want = 0.0
    for l in range(L):
        if scope == VECTOR:
            groups = [(slice(0, sizes[l]), float(np.sqrt(sum(np.sum(a.astype(np.float64) ** 2) for a in g))))]
        else:
            groups = [(slice(b, min(b + 128, sizes[l])), float(np.sqrt(np.sum(g[l][b: b + 128].astype(np.float64) ** 2))))
                      for b in range(0, sizes[l], 128)]
        for sl, norm in groups:
            u = np.abs(g[l][sl].astype(np.float64)) / norm
            tau = np.clip(np.searchsorted(lev.astype(np.float64), u, side="right") - 1, 0, S - 2)
            var = norm ** 2 * (lev[tau + 1] - u) * (u - lev[tau])
            want += float(np.sum(var))
            sd = np.sqrt(var / seeds)
            assert np.all(np.abs(mean[l][sl] / seeds - g[l][sl]) <= 5 * sd + 1e-6 * norm)
    assert err2 / seeds == pytest.approx(want, rel=0.03)


def test_on_grid_values_are_reproduced_in_every_bucket(oracle):
    """u on a level is reproduced exactly whatever the draw: buckets whose single non-zero entry carries the norm
    (u = 1 there, u = 0 elsewhere), each bucket with a different power-of-two norm, both signs."""
    S = 5
    lev = np.array([0.0, 0.25, 0.5, 0.75, 1.0], np.float32)
    d = 128 * 6
    v = np.zeros(d, np.float32)
    for b in range(6):
        v[128 * b + 17 * b] = 2.0 ** b * (-1) ** b
    for seed in range(5):
        msg, _, _, _ = oracle.quantize([d], [S], [lev], [v], seed, 1, 0, scope=BUCKET)
        assert np.array_equal(_decode_layers(oracle, [d], S, msg, BUCKET)[0], v)


def test_previous_message_distance_in_bucket_scope(oracle):
    S, sizes = 8, [3000, 129]
    lev1, lev2 = uniform_levels(S), np.array([0, .02, .05, .1, .2, .4, .7, 1.0], np.float32)
    rng = np.random.default_rng(7)
    g1 = [rng.standard_normal(s).astype(np.float32) for s in sizes]
    g2 = [rng.standard_normal(s).astype(np.float32) * 2 for s in sizes]
    m1, _, _, _ = oracle.quantize(sizes, [S] * 2, [lev1] * 2, g1, 9, 1, 0, scope=BUCKET)
    m2, _, d2, _ = oracle.quantize(sizes, [S] * 2, [lev2] * 2, g2, 9, 2, 0, msg_prev=m1, scope=BUCKET)
    a = _decode_layers(oracle, sizes, S, m1, BUCKET)
    b = _decode_layers(oracle, sizes, S, m2, BUCKET)
    want = sum(float(np.sum((x.astype(np.float64) - y) ** 2)) for x, y in zip(b, a))
    assert d2 == pytest.approx(want, rel=1e-5)
    assert oracle.delta_from_messages(sizes, [S] * 2, m2, m1, scope=BUCKET) == d2


def test_fit_pooled_weights_from_the_definition(oracle):
    """Bucket scope: W[bin(u)] += floor(sumsq_b * 2^(23 - e)) over every coordinate, recomputed with numpy;
    vector scope with one layer equals the per-layer fit."""
    S, K = 8, 2
    sizes = [5000, 1300]
    rng = np.random.default_rng(8)
    g = [[(rng.standard_t(3, s) * 10.0 ** rng.uniform(-3, 1)).astype(np.float32) for s in sizes] for _ in range(K)]
    flat = [g[k][l] for k in range(K) for l in range(len(sizes))]
    lev0 = [uniform_levels(S)]
    lev, _, pooled, st = oracle.fit_levels(sizes, [0, 0], [S], K, flat, lev0, scope=BUCKET)
    assert st == 0
    sums = {}
    smax = 0.0
    for k in range(K):
        for l, s in enumerate(sizes):
            for b in range(0, s, 128):
                sums[(k, l, b)] = oracle.bucket_sumsq(g[k][l][b: b + 128])
                smax = max(smax, sums[(k, l, b)])            # the scale comes from the heaviest bucket
    ex = int(np.floor(np.log2(smax)))
    W = np.zeros(257, dtype=np.uint64)
    for (k, l, b), sv in sums.items():
        wfix = int(np.floor(np.ldexp(sv, 23 - ex)))
        inv = oracle.rcp_floor(oracle.sqrt_floor(sv))
        if wfix == 0 or inv == 0:
            continue
        seg = g[k][l][b: b + 128]
        seg = seg[((seg.view(np.uint32) & 0x7FFFFFFF) >> 20) != 0]
        u = np.minimum(np.abs(seg) * np.float32(inv), np.float32(1.0)).astype(np.float32)
        j = np.clip((u.view(np.uint32) >> 20).astype(np.int64) - 760, 0, 256)
        np.add.at(W, j, np.uint64(wfix))
    assert np.array_equal(pooled[0], W)
    assert np.array_equal(lev[0], oracle.fit_dp(W, S))
    # weights follow the buckets' squared norms: the heaviest bucket's bins dominate the total
    assert pooled[0].sum() > 0
    one = [g[0][0]]
    a, _, pa, _ = oracle.fit_levels([sizes[0]], [0], [S], 1, one, lev0, scope=LAYER)
    b, _, pb, _ = oracle.fit_levels([sizes[0]], [0], [S], 1, one, lev0, scope=VECTOR)
    assert np.array_equal(pa, pb) and np.array_equal(a[0], b[0])


def test_fit_lowers_the_variance_in_bucket_scope(oracle):
    """End to end: levels fitted in bucket scope beat uniform levels on the exact variance eq. (Var) with bucket norms."""
    S, K = 8, 2
    w = workloads.get("dcgan")
    sizes = [20000]
    g = [workloads.layer_numpy(w, 1, k, 1)[:20000].copy() for k in range(K)]
    lev, _, _, _ = oracle.fit_levels(sizes, [0], [S], K, g, [uniform_levels(S)], scope=BUCKET)

    def exact_var(levels):
        levels = levels.astype(np.float64)
        tot = 0.0
        for a in g:
            for b in range(0, a.size, 128):
                seg = a[b: b + 128].astype(np.float64)
                n = np.sqrt(np.sum(seg ** 2))
                if n == 0:
                    continue
                u = np.abs(seg) / n
                tau = np.clip(np.searchsorted(levels, u, side="right") - 1, 0, S - 2)
                tot += n ** 2 * float(np.sum((levels[tau + 1] - u) * (u - levels[tau])))
        return tot

    assert exact_var(lev[0]) < 0.8 * exact_var(uniform_levels(S))


def test_statistics_gathered_while_quantizing_equal_the_explicit_fit(oracle):
    """Alg. 1 updates the levels before the round's vectors exist, so the estimate comes from the previous round:
    the pass that quantizes (bucket scope) gathers the same pooled weights as the explicit fit on those vectors when it
    is given the same scale, and the fit from the gathered statistics gives the same levels; the scale it hands on is
    the exponent of the largest bucket sum; without a scale nothing is gathered and the levels stay."""
    S, K = 8, 2
    sizes, types = [5000, 1300, 0, 70000], [0, 0, 1, 1]
    L = len(sizes)
    rng = np.random.default_rng(9)
    g = [[(rng.standard_t(3, s) * 10.0 ** rng.uniform(-3, 1)).astype(np.float32) for s in sizes] for _ in range(K)]
    flat = [g[k][l] for k in range(K) for l in range(L)]
    lev0 = [uniform_levels(S), uniform_levels(S)]
    want_lev, _, want_pooled, _ = oracle.fit_levels(sizes, types, [S, S], K, flat, lev0, scope=BUCKET)
    # the explicit fit's scale: exponent of the largest bucket sum of the type
    exps = []
    for m in range(2):
        smax = 0.0
        for k in range(K):
            for l in range(L):
                if types[l] != m:
                    continue
                for b in range(0, sizes[l], 128):
                    smax = max(smax, oracle.bucket_sumsq(g[k][l][b: b + 128]))
        exps.append(int(np.floor(np.log2(smax))))
    lev_l = [lev0[types[l]] for l in range(L)]
    hist = np.zeros((K, L, 257), np.uint64)
    bmax = np.zeros((K, L))
    for k in range(K):
        plain = oracle.quantize(sizes, [S] * L, lev_l, g[k], 5, 1, k, scope=BUCKET)
        out = oracle.quantize(sizes, [S] * L, lev_l, g[k], 5, 1, k, scope=BUCKET, stats_exp=[exps[t] for t in types])
        assert np.array_equal(plain[0], out[0]) and plain[2] == out[2]          # gathering does not change the message
        hist[k], bmax[k] = out[4], out[5]
    lev, pooled, new_exps, st = oracle.fit_from_stats(types, [S, S], K, hist, bmax, exps, lev0)
    assert st == 0 and np.array_equal(pooled, want_pooled)
    assert all(np.array_equal(a, b) for a, b in zip(lev, want_lev))
    assert list(new_exps) == exps
    # no scale yet: nothing gathered, levels kept, but the next scale is produced
    out = oracle.quantize(sizes, [S] * L, lev_l, g[0], 5, 1, 0, scope=BUCKET, stats_exp=[oracle.TYPE_SKIP] * L)
    assert out[4].sum() == 0 and out[5].max() > 0
    h1 = np.zeros((K, L, 257), np.uint64)
    lev, pooled, e2, _ = oracle.fit_from_stats(types, [S, S], K, h1, bmax, [oracle.TYPE_SKIP] * 2, lev0)
    assert all(np.array_equal(a, b) for a, b in zip(lev, lev0)) and list(e2) == exps
    # a scale from an earlier, much smaller round: weights hit the cap 2^30 instead of overflowing
    out = oracle.quantize(sizes, [S] * L, lev_l, g[0], 5, 1, 0, scope=BUCKET, stats_exp=[e - 40 for e in [exps[t] for t in types]])
    assert (1 << 30) <= int(out[4].max()) and int(out[4].sum()) <= sum(sizes) * (1 << 30)
