"""qoda_quantize_noalloc (the entry point for callers that cannot allocate) against qoda_quantize, through the C ABI:
same message bytes and the same step-size term, on two calls in a row, the second with a smaller model -- the static
scratch still holds the first call's contents then.  Layer, vector and bucket scope."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2505_14371_amd import qoda, workloads  # noqa: E402


def _model(sizes, S, K, seed, scope):
    dev = torch.device("cuda:0")
    L = len(sizes)
    ctx = qoda.Context(sizes, list(range(L)), [S] * L, K, seed, norm_scope=scope)
    off, n = workloads.padded_offsets(sizes)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    grads = []
    for k in range(K):
        z = torch.randn((4, n), device=dev, generator=gen)
        grads.append((z[0] / torch.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0) * 1e-3).contiguous())
    mb = ctx.message_bytes()
    new = lambda: [torch.full((mb,), 0xA5, dtype=torch.uint8, device=dev) for _ in range(K)]
    return ctx, off, grads, new


def _two_rounds(ctx, off, grads, new, K, call):
    """Two rounds (the second against the first round's message) with ``call`` as the quantize entry point."""
    msgs = [new(), new()]
    deltas = []
    for t in (1, 2):
        cur = (t - 1) & 1
        for k in range(K):
            ptrs = [grads[(k + t) % K].data_ptr() + 4 * int(o) for o in off]
            call(k, ptrs, t, msgs[cur][k], msgs[1 - cur][k] if t > 1 else None)
        deltas.append(ctx.read_buffer(qoda.BUF_DELTA).copy())
    torch.cuda.synchronize()
    assert ctx.status() == qoda.OK
    return [[m.cpu().numpy() for m in ms] for ms in msgs], deltas


@pytest.mark.parametrize("scope", [qoda.SCOPE_LAYER, qoda.SCOPE_VECTOR, qoda.SCOPE_BUCKET])
def test_noalloc_quantize_matches_quantize_on_two_calls_in_a_row(scope):
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    big = [16384 * 5 + 1237, 410, 0, 2100, 16384 * 2, 70001]      # several tiles, ragged tails, an empty layer
    small = [3000, 257, 16384 + 5]                               # fewer and smaller layers: stale scratch beyond them
    for sizes, S, K, seed in ((big, 8, 3, 11), (small, 16, 2, 12)):
        ctx, off, grads, new = _model(sizes, S, K, seed, scope)
        want_msgs, want_deltas = _two_rounds(ctx, off, grads, new, K, ctx.quantize)
        got_msgs, got_deltas = _two_rounds(ctx, off, grads, new, K, ctx.quantize_noalloc)
        for t in range(2):
            assert np.array_equal(got_deltas[t], want_deltas[t]), (sizes, t)
            for k in range(K):
                assert np.array_equal(got_msgs[t][k], want_msgs[t][k]), (sizes, t, k)
        ctx.close()


def test_noalloc_quantize_rejects_models_beyond_the_static_scratch():
    if not torch.cuda.is_available():
        pytest.fail("a GPU test was selected but no GPU is visible")
    dev = torch.device("cuda:0")
    L = 4097                                                     # one layer more than the scratch holds
    ctx = qoda.Context([4] * L, [0] * L, [4], 1, 1)
    g = torch.zeros(64 * L, dtype=torch.float32, device=dev)
    msg = torch.zeros(ctx.message_bytes(), dtype=torch.uint8, device=dev)
    with pytest.raises(qoda.QodaError) as e:
        ctx.quantize_noalloc(0, [g.data_ptr() + 256 * l for l in range(L)], 1, msg)
    assert e.value.code == qoda.EINVAL and "static scratch" in str(e.value)
    ctx.close()
