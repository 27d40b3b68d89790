"""The contract's narrowed arithmetic bounded against the plain definitions (oracle: "plain definitions" section).

Three quantities of the bit-level contract are cheaper than their textbook definition: the step-size term of
eq. (general_stepsize) (single-precision chains inside a reduction slot), the bucket sum of squares of the bucket
scope (single-precision chains inside a lane, exact fp64 when the result leaves a safe range), and the level fit
(a histogram of every coordinate on a 1/8-octave grid instead of the samples themselves).  Each is compared here with
the definition written out in fp64, within a bound derived from the arithmetic, and the property the paper needs from
it (a step size, u <= 1 and E[Q(v)] = v of Thm 5.1, a small objective eq. (MQV)) is checked directly."""
import numpy as np
import pytest

from paper_2505_14371_amd import workloads

LAYER, VECTOR, BUCKET = 0, 1, 2
EPS = 2.0 ** -24                      # one fp32 rounding


def uniform_levels(S):
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


def ulps_apart(a, b):
    return abs(int(np.float32(a).view(np.int32)) - int(np.float32(b).view(np.int32)))


# ------------------------------------------------------------------------------------------ the step-size term
# A slot adds at most 64 non-negative terms with one rounding each (fused multiply-add): relative error at most
# 64 * 2^-24 of the slot's sum; each term's difference cur - prev is one fp32 subtraction: 2 * 2^-24 on its square;
# everything above the slots is fp64.  Terms below 2^-126 lose absolute 2^-150 each.
DELTA_REL_BOUND = 66 * EPS


@pytest.mark.parametrize("name", ["bilinear", "microbench", "dcgan", "txl", "gpt1p3b"])
def test_step_size_term_against_the_fp64_definition(oracle, name):
    w = workloads.mini(name, max_layer=60000, max_layers=6)
    L, S, K = len(w.sizes), w.points, 2
    lev = [uniform_levels(S)] * L
    prev = [None] * K
    acc_c = acc_p = 0.0
    for t in (1, 2, 3):
        dc, dp = [], []
        for k in range(K):
            g = workloads.node_numpy(w, k, t)
            m, _, d, st = oracle.quantize(w.sizes, [S] * L, lev, g, w.seed, t, k, msg_prev=prev[k])
            assert st == 0
            p = oracle.delta_plain(w.sizes, [S] * L, m, prev[k])
            # the plain routine against numpy on the decoded vectors (eq. (general_stepsize), one node's term)
            cur = oracle.dequant_aggregate(w.sizes, [S] * L, [m])
            old = oracle.dequant_aggregate(w.sizes, [S] * L, [prev[k]]) if prev[k] is not None else [np.zeros_like(a) for a in cur]
            want = sum(float(np.sum((a.astype(np.float64) - b.astype(np.float64)) ** 2)) for a, b in zip(cur, old))
            assert p == pytest.approx(want, rel=1e-12)
            assert abs(d - p) <= DELTA_REL_BOUND * p + w.total * 2.0 ** -150, (t, k)
            dc.append(d)
            dp.append(p)
            prev[k] = m
        # the step size that each accumulator yields: the same float, or its neighbour
        acc_c, eta_c = oracle.step_size(dc, acc_c)
        acc_p, eta_p = oracle.step_size(dp, acc_p)
        assert ulps_apart(eta_c, eta_p) <= 1, t
        # worst case of the bound above: d(eta)/eta = -(1/2) d(acc)/(1 + acc)
        assert abs(float(eta_c) - float(eta_p)) <= (0.5 * DELTA_REL_BOUND + 2 * EPS) * float(eta_p)


def test_step_size_term_bound_holds_for_an_adversarial_slot(oracle):
    """One large term followed by 63 terms that each fall just below half a unit in the last place of the running sum:
    a single-precision chain drops every one of them.  The loss stays inside the derived bound."""
    d = 16384
    v = np.zeros(d, np.float32)
    slot = np.arange(0, d, 256)                    # coordinates 0, 256, ...: the 64 terms of slot 0 of the chunk
    lev = np.array([0.0, 2.0 ** -12.1, 1.0], np.float32)
    # on-grid values decode exactly: the vector's norm is (about) 1, entries 1 and 63 times the small level
    v[slot[0]] = 1.0
    v[slot[1:]] = lev[1]
    m, ss, dc, st = oracle.quantize([d], [3], [lev], [v], 1, 1, 0)
    dp = oracle.delta_plain([d], [3], m)
    assert st == 0 and dp > 0
    rel = abs(dc - dp) / dp
    assert 0.2 * EPS < rel <= DELTA_REL_BOUND      # the chain does lose something here, and no more than allowed


# ------------------------------------------------------------------------------------------ bucket sums of squares
# A lane adds 4 squares with one rounding each: relative error at most 4 * 2^-24 as long as no square is lost, which
# the rule "below 2^-100 or not finite -> exact fp64 squares" guarantees to 2^-42; the tree above the lanes is fp64.
def test_bucket_sum_against_the_fp64_definition_over_the_whole_float_range(oracle):
    rng = np.random.default_rng(5)
    for trial in range(400):
        n = int(rng.integers(1, 129))
        scale = 10.0 ** rng.uniform(-44, 18.5)
        v = (rng.standard_t(3, n) * scale).astype(np.float32)
        if rng.random() < 0.3:                     # a bucket dominated by one entry
            v[rng.integers(0, n)] = np.float32(min(scale * 1e4, 1e19))
        plain = oracle.sumsq_plain(v)
        assert plain == pytest.approx(float(np.sum(v.astype(np.float64) ** 2)), rel=1e-13, abs=0.0)
        got = oracle.bucket_sumsq(v)
        assert abs(got - plain) <= (4 * EPS + 2.0 ** -40) * plain, (trial, scale)
        # what Thm 5.1 needs from the norm: no entry exceeds it by more than a rounding, so u = |v| / norm is not cut
        # by the clamp at 1 (a norm that is too small would bias the largest entry)
        norm = float(oracle.sqrt_floor(got))
        assert norm >= float(np.abs(v).max()) * (1 - 3 * EPS)
        assert norm <= np.sqrt(plain) * (1 + 3 * EPS)


def expectation_of_Q(oracle, v, inv, norm, lev):
    """E[Q(v_i)] over all 65536 equally likely draws, per coordinate (Sec. 3.1), by enumeration."""
    draws = np.arange(65536, dtype=np.uint32)
    out = np.zeros(v.size)
    for i in range(v.size):
        sign, idx = oracle.quantize_with_draws(np.full(65536, v[i], np.float32), inv, lev, draws)
        out[i] = float(np.mean(oracle.decode(sign, idx, norm, lev).astype(np.float64)))
    return out


@pytest.mark.parametrize("scale", [1e-25, 3e-30, 1e-36, 1e19])
def test_buckets_outside_the_single_precision_range_stay_unbiased(oracle, scale):
    """A bucket whose squares vanish (or overflow) in single precision: the message decodes to an unbiased estimate of
    the bucket all the same (Thm 5.1), because its norm comes from exact fp64 squares then."""
    rng = np.random.default_rng(2)
    S = 8
    lev = uniform_levels(S)
    v = (rng.standard_normal(128) * scale).astype(np.float32)
    msg, _, _, st = oracle.quantize([128], [S], [lev], [v], 3, 1, 0, scope=BUCKET)
    assert st == 0
    sign, idx, norms = oracle.unpack_layer(msg[oracle.header_bytes([128], [S], BUCKET):], 128, S, BUCKET)
    norm = float(norms[0])
    assert norm == pytest.approx(float(np.sqrt(np.sum(v.astype(np.float64) ** 2))), rel=4 * EPS)
    pick = np.array([0, 17, int(np.argmax(np.abs(v))), int(np.argmin(np.abs(v)))])
    e = expectation_of_Q(oracle, v[pick], oracle.rcp_floor(norm), norm, lev)
    gap = norm / (S - 1)
    assert np.all(np.abs(e - v[pick].astype(np.float64)) <= gap * 2.0 ** -16 + np.abs(v[pick]) * 4 * EPS)
    # and the decoded message is exactly +-norm * level
    dec = oracle.dequant_aggregate([128], [S], [msg], scope=BUCKET)[0]
    assert np.array_equal(dec, np.where(sign == 1, -1.0, 1.0).astype(np.float32) * (np.float32(norm) * lev[idx]))


@pytest.mark.parametrize("scope", [LAYER, VECTOR, BUCKET])
def test_a_norm_below_the_normal_range_is_flagged(oracle, scope):
    """0 < norm < 2^-126: 1/norm is not a float, the reciprocal is cut at FLT_MAX and u = |v| * inv falls short of
    |v| / norm -- the one case where E[Q(v)] = v fails; it raises a status bit of its own."""
    S = 4
    lev = uniform_levels(S)
    v = np.zeros(300, np.float32)
    v[:128] = np.float32(1e-41)                    # subnormal entries: the norm of this vector / bucket is about 1e-40
    _, _, _, st = oracle.quantize([300], [S], [lev], [v], 1, 1, 0, scope=scope)
    assert st == 2
    v[:128] = np.float32(1e-37)                    # norm about 1e-36: fine
    _, _, _, st = oracle.quantize([300], [S], [lev], [v], 1, 1, 0, scope=scope)
    assert st == 0
    v[200] = np.inf
    _, _, _, st = oracle.quantize([300], [S], [lev], [v], 1, 1, 0, scope=scope)
    assert st & 1


# ------------------------------------------------------------------------------------------ the level fit
def structured_layers():
    rng = np.random.default_rng(4)
    t = rng.standard_t(3, size=(128, 2048))
    cols = np.arange(2048)
    return {
        "sorted by magnitude": np.sort(np.abs(t.ravel())).astype(np.float32),
        "column scales ramp": (t * 10.0 ** np.linspace(-2, 0, 2048)).astype(np.float32).ravel(),
        "every fourth column block cold": (t * np.where((cols // 256) % 4 == 0, 0.01, 1.0)).astype(np.float32).ravel(),
        "every fourth column block hot": (t * np.where((cols // 256) % 4 == 0, 1.0, 0.01)).astype(np.float32).ravel(),
    }


@pytest.mark.parametrize("scope", [LAYER, BUCKET])
def test_the_estimate_does_not_depend_on_where_a_coordinate_sits(oracle, scope):
    """Alg. 1 line 4 estimates the distribution of the normalised coordinates: a property of the multiset of values (of
    the multiset of buckets under bucket scope), not of their positions.  Every coordinate is counted, so layers with
    structure along the index (sorted values, hot and cold column blocks of a weight matrix) are fitted as well as
    their shuffles: the objective eq. (MQV) of the fitted levels is the same up to rounding of the norms."""
    rng = np.random.default_rng(6)
    for name, v in structured_layers().items():
        if scope == BUCKET:                        # shuffle whole buckets: the multiset of buckets is what counts
            perm = (rng.permutation(v.size // 128)[:, None] * 128 + np.arange(128)[None, :]).ravel()
        else:
            perm = rng.permutation(v.size)
        shuffled = v[perm]
        for S in (4, 8, 16):
            a, _, pa, _ = oracle.fit_levels([v.size], [0], [S], 1, [v], [uniform_levels(S)], scope=scope)
            b, _, pb, _ = oracle.fit_levels([v.size], [0], [S], 1, [shuffled], [uniform_levels(S)], scope=scope)
            assert pa.sum() == pytest.approx(pb.sum(), rel=1e-6)
            fa = oracle.mqv_objective_plain([v.size], [0], [S], 1, [v], a, scope=scope)
            fb = oracle.mqv_objective_plain([v.size], [0], [S], 1, [v], b, scope=scope)
            assert fa == pytest.approx(fb, rel=1e-3), (name, S)


def test_mqv_objective_routine_against_numpy(oracle):
    w = workloads.mini("txl", max_layer=5000, max_layers=3)
    K, L, S = 2, 3, 8
    g = [workloads.layer_numpy(w, k, l, 1) for k in range(K) for l in range(L)]
    lev = np.array([0, 0.01, 0.03, 0.07, 0.15, 0.3, 0.6, 1.0], np.float32)

    def var(vec, norm):
        u = np.minimum(np.abs(vec.astype(np.float64)) / norm, 1.0)
        lv = lev.astype(np.float64)
        tau = np.clip(np.searchsorted(lv, u, side="right") - 1, 0, S - 2)
        return norm ** 2 * float(np.sum((lv[tau + 1] - u) * (u - lv[tau])))

    n2 = lambda a: float(np.sqrt(np.sum(a.astype(np.float64) ** 2)))
    want = {LAYER: sum(var(a, n2(a)) for a in g),
            VECTOR: sum(var(g[k * L + l], n2(np.concatenate(g[k * L: (k + 1) * L]))) for k in range(K) for l in range(L)),
            BUCKET: sum(var(a[b: b + 128], n2(a[b: b + 128])) for a in g for b in range(0, a.size, 128))}
    for scope in (LAYER, VECTOR, BUCKET):
        got = oracle.mqv_objective_plain(w.sizes, [0] * L, [S], K, g, [lev], scope=scope)
        assert got == pytest.approx(want[scope], rel=1e-10)
    assert oracle.variance_plain(g[0], lev) == pytest.approx(var(g[0], n2(g[0])), rel=1e-12)


@pytest.mark.parametrize("scope", [LAYER, VECTOR, BUCKET])
@pytest.mark.parametrize("name", ["dcgan", "txl", "gpt1p3b"])
def test_histogram_objective_tracks_the_objective_on_the_samples(oracle, name, scope):
    """The fit minimises eq. (Qada2) with the mass of every 1/8-octave bin placed at its midpoint.  For levels that are
    many bins apart (uniform ones) that histogram objective equals eq. (MQV) evaluated on the samples themselves within
    a few per cent.  Where two fitted levels are neighbouring grid points the midpoint carries the largest variance the
    bin can have, (w/2)^2 against w^2/6 for mass spread evenly over a bin of width w: the histogram objective then
    overstates the true one, by at most that factor 3/2.  The fitted levels are far better than uniform ones on the
    true objective."""
    w = workloads.mini(name, max_layer=40000, max_layers=5)
    K, L, S = 2, len(w.sizes), w.points
    g = [workloads.layer_numpy(w, k, l, 1) for k in range(K) for l in range(L)]
    types = [0] * L if scope == VECTOR else list(range(L))
    M = max(types) + 1
    lev, _, pooled, st = oracle.fit_levels(w.sizes, types, [S] * M, K, g, [uniform_levels(S)] * M, scope=scope)
    assert st == 0
    true_fit = oracle.mqv_objective_plain(w.sizes, types, [S] * M, K, g, lev, scope=scope)
    true_uni = oracle.mqv_objective_plain(w.sizes, types, [S] * M, K, g, [uniform_levels(S)] * M, scope=scope)
    assert true_fit < 0.5 * true_uni
    if scope == LAYER:                             # one type per layer: the histogram objective per type, rescaled
        for l in range(L):
            smax = max(oracle.sumsq(g[k * L + l]) for k in range(K))
            scale = 2.0 ** (23 - int(np.floor(np.log2(smax))))
            for levels, hi in ((lev[l], 1.5), (uniform_levels(S), 1.05)):
                est = oracle.fit_objective(pooled[l], levels) / scale
                true = oracle.mqv_objective_plain([w.sizes[l]], [0], [S], K, [g[k * L + l] for k in range(K)], [levels])
                assert 0.95 * true <= est <= hi * true, (l, S, est / true)


def test_one_interior_level_is_within_the_grid_step_of_the_true_optimum(oracle):
    """S = 3: the single interior level can be optimised by brute force on the samples (eq. (MQV) is a function of one
    variable); the fitted grid level gives an objective within 2 % of that optimum."""
    w = workloads.get("dcgan")
    v = workloads.layer_numpy(w, 0, 3, 1)[:60000].copy()
    lev, _, _, _ = oracle.fit_levels([v.size], [0], [3], 1, [v], [uniform_levels(3)])
    got = oracle.variance_plain(v, lev[0])
    best = min(oracle.variance_plain(v, np.array([0.0, x, 1.0], np.float32)) for x in np.geomspace(1e-4, 0.9, 400))
    assert got <= 1.02 * best
