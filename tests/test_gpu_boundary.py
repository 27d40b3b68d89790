"""Behaviour of the C-ABI boundary that a caller can trip over: which norms a quantize call uses after a fit, host
arrays that change right after a call, and per-node calls that never wait for an upload."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import helpers  # noqa: E402
from paper_2505_14371_amd import qoda, workloads  # noqa: E402


def gm(*a, **k):
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    import gpu_harness

    return gpu_harness.GpuModel(*a, **k)


def _vectors(w, K, t):
    return [workloads.node_numpy(w, k, t) for k in range(K)]


@pytest.mark.parametrize("per_node", [False, True])
def test_vectors_rewritten_between_fit_and_quantize_are_quantized_with_their_own_norms(oracle, per_node):
    """Alg. 1 updates the levels (lines 3-5) before the round's vectors exist (line 11): a caller in that order fits on
    the earlier vectors, then writes the round's vectors into the SAME buffers, then quantizes with the same round
    number.  qoda_fit_levels leaves nothing behind that such a call could mistake for the new vectors' norms."""
    w = workloads.mini("dcgan", max_layer=30000, max_layers=5)
    L, K, S = len(w.sizes), 3, w.points
    m = gm(w.sizes, list(range(L)), [S] * L, K, seed=w.seed)
    old, new = _vectors(w, K, 1), [[(3.0 * a).astype(np.float32) for a in g] for g in _vectors(w, K, 2)]
    m.set_grads(old)
    m.fit(2)                                                     # qoda_fit_levels on the earlier vectors, round 2
    m.set_grads(new)                                             # same buffers, new contents
    if per_node:
        m.quantize_each(2)
    else:
        m.quantize_all(2)
    msgs = m.messages()
    flat = [old[k][l] for k in range(K) for l in range(L)]
    lev, _, _, _ = oracle.fit_levels(w.sizes, list(range(L)), [S] * L, K, flat, [helpers.uniform_levels(S)] * L)
    for k in range(K):
        want, _, _, st = oracle.quantize(w.sizes, [S] * L, lev, new[k], w.seed, 2, k)
        assert st == 0 and np.array_equal(msgs[k], want), k


def test_kept_norms_are_used_only_for_the_declared_round_and_pointers(oracle):
    """qoda_fit_levels_keep_norms declares "these are the round's vectors": the quantize call of that round with those
    pointers skips its norm pass.  The declaration is the caller's: rewriting the buffers in between yields messages
    scaled by the stale norms (shown here on purpose); another round number drops the kept norms."""
    w = workloads.mini("txl", max_layer=30000, max_layers=4)
    L, K, S = len(w.sizes), 2, w.points
    m = gm(w.sizes, list(range(L)), [S] * L, K, seed=w.seed)
    g1 = _vectors(w, K, 1)
    g2 = [[(5.0 * a).astype(np.float32) for a in g] for g in _vectors(w, K, 2)]
    flat = [g1[k][l] for k in range(K) for l in range(L)]
    lev, _, _, _ = oracle.fit_levels(w.sizes, list(range(L)), [S] * L, K, flat, [helpers.uniform_levels(S)] * L)
    want1 = [oracle.quantize(w.sizes, [S] * L, lev, g1[k], w.seed, 1, k)[0] for k in range(K)]
    want2 = [oracle.quantize(w.sizes, [S] * L, lev, g2[k], w.seed, 1, k)[0] for k in range(K)]
    # kept and used as declared: no norm pass runs in the quantize call
    m.set_grads(g1)
    m.ctx.fit_levels_keep_norms(m.grad_ptrs(), 1)
    m.ctx.profile_enable(True)
    m.quantize_all(1)
    m.sync()
    assert "k_sumsq<false>" not in m.ctx.profile_read()
    assert all(np.array_equal(a, b) for a, b in zip(m.messages(), want1))
    # the declaration broken by the caller: stale norms, and the library cannot tell
    m.ctx.fit_levels_keep_norms(m.grad_ptrs(), 1)
    m.set_grads(g2)
    m.quantize_all(1)
    m.sync()
    assert not all(np.array_equal(a, b) for a, b in zip(m.messages(), want2))
    # another round number: the kept norms are not used
    m.set_grads(g1)
    m.ctx.fit_levels_keep_norms(m.grad_ptrs(), 1)
    m.set_grads(g2)
    m.ctx.profile_read()
    m.quantize_all(2)
    m.sync()
    assert "k_sumsq<false>" in m.ctx.profile_read()
    want = [oracle.quantize(w.sizes, [S] * L, lev, g2[k], w.seed, 2, k)[0] for k in range(K)]
    assert all(np.array_equal(a, b) for a, b in zip(m.messages(), want))
    m.ctx.profile_enable(False)


def test_host_arrays_may_change_as_soon_as_a_call_returns(oracle):
    """Pointer arrays and level values are consumed inside the call (they travel as kernel arguments): a caller may
    overwrite them at once, long before the device gets to the work."""
    w = workloads.mini("txl", max_layer=50000, max_layers=6)
    L, K, S = len(w.sizes), 2, w.points
    m = gm(w.sizes, [0] * L, [S], K, seed=w.seed)
    g = _vectors(w, K, 1)
    m.set_grads(g)
    lev = np.array([0, 0.01, 0.03, 0.07, 0.15, 0.3, 0.6, 1.0], np.float32)
    # a long-running kernel first, so that everything below is still queued when the host arrays are trashed
    busy = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
    for _ in range(8):
        busy.normal_()
    lv = lev.copy()
    m.ctx.set_levels(0, lv)
    lv[:] = 0.5
    gp = qoda.pointer_array(m.grad_ptrs())
    mp = qoda.pointer_array(m.msg[m.cur])
    m.ctx.quantize_all(gp, 1, mp, None)
    for i in range(len(gp)):
        gp[i] = 0
    for i in range(len(mp)):
        mp[i] = 0
    m.sync()
    for k in range(K):
        want = oracle.quantize(w.sizes, [S] * L, [lev] * L, g[k], w.seed, 1, k)[0]
        assert np.array_equal(m.messages()[k], want), k
    assert m.ctx.status() == qoda.OK
