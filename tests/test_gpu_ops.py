"""Operator-level parity: each HIP kernel, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Shapes span several tiles and ragged tails; widths follow the row-kernel
extents the paper targets (Section 2.2: hidden up to 12288/16384, sequence up to 4096)."""
import numpy as np
import pytest
import torch

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl
from tests.gpu_util import dev, gate, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


# fp16 rounding of an O(1) output: half an ulp at |x| in [2,4) is 1e-3; budget a few of them
OP_MAX, OP_MEAN = 6e-3, 6e-4


@pytest.mark.parametrize("rows,width", [(7, 64), (5, 768), (3, 1024), (3, 1280), (2, 2048), (3, 4096), (2, 12288),
                                        (2, 16384), (2, 49152), (4, 100), (3, 1283), (300, 1024),
                                        # 64 rows and more, up to 2048 wide: one wave per row, four rows per workgroup
                                        (67, 64), (301, 768), (130, 1280), (65, 2048), (64, 8), (3150, 1024)])
def test_layernorm(eet, rows, width):
    x = (wl.normal(101, width, (rows, width)).astype(np.float32) * 1.7 + 0.3).astype(np.float16)
    g = wl.normal(102, width, (width,), 0.1, 1.0)
    b = wl.normal(103, width, (width,), 0.1, 0.0)
    y = torch.full((rows, width), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_layernorm(dev(x), dev(g), dev(b), y, 1e-5)
    torch.cuda.synchronize()
    gate(host(y), orc.layernorm(x, g, b, 1e-5), f"layernorm {rows}x{width}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("S,lens", [(64, [64, 17]), (520, [333, 520]), (9, [9, 4])])
def test_softmax_maskfree_with_scores_that_leave_one_key_standing(eet, S, lens):
    """Scores with a standard deviation of 30 and a scale of 1: every row is close to one-hot, most probabilities
    underflow, none may overflow or turn into NaN, and rows still sum to one."""
    B = len(lens)
    s = (wl.scores(29, B, 2, S).astype(np.float32) * 15.0).astype(np.float16)
    sd = dev(s)
    eet.eet_op_softmax_maskfree(sd, lens, 1.0)
    torch.cuda.synchronize()
    got, want = host(sd), orc.softmax_maskfree(s, lens, 1.0)
    for b, L in enumerate(lens):
        gate(got[b, :, :L], want[b, :, :L], f"one-hot softmax b={b}", 1e-3, 1e-4)
        np.testing.assert_allclose(got[b, :, :L].astype(np.float64).sum(-1), 1.0, atol=2e-3)


@pytest.mark.parametrize("rows,width", [(3, 1024), (70, 768), (2, 4096), (3, 1283)])
def test_layernorm_of_constant_rows_gives_beta(eet, rows, width):
    """Zero variance: the result is beta exactly (the deviations are exact zeros; eps keeps the scale finite)."""
    x = np.full((rows, width), 0.1, np.float16)
    x[1] = 1.5
    x[-1] = -7.0
    g = wl.normal(102, width, (width,), 0.1, 1.0)
    b = wl.normal(103, width, (width,), 0.1, 0.0)
    y = torch.full((rows, width), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_layernorm(dev(x), dev(g), dev(b), y, 1e-5)
    torch.cuda.synchronize()
    assert np.array_equal(host(y), np.broadcast_to(b, (rows, width)))


@pytest.mark.parametrize("rows,width", [(5, 1024), (130, 1024), (3, 4096), (2, 12288), (3, 1283)])
def test_layernorm_of_rows_with_a_large_mean_and_an_outlier(eet, rows, width):
    """Rows whose mean is a hundred standard deviations away from zero (a one-pass variance would cancel), and rows with
    one element a thousand times the others (the statistics are then that element's)."""
    base = wl.normal(105, width, (rows, width)).astype(np.float32)
    shifted = (base + 100.0).astype(np.float16)
    spiked = base.copy()
    spiked[:, 0] = 1000.0
    spiked[1:, 0] = 0.1
    spiked[1:, width // 2] = -3000.0
    spiked = spiked.astype(np.float16)
    g = np.ones(width, np.float16)
    b = np.zeros(width, np.float16)
    for name, x in (("mean 100", shifted), ("spike", spiked)):
        y = torch.full((rows, width), float("nan"), dtype=torch.float16, device="cuda:0")
        eet.eet_op_layernorm(dev(x), dev(g), dev(b), y, 1e-5)
        torch.cuda.synchronize()
        want = orc.layernorm(x, g, b, 1e-5)
        got = host(y).astype(np.float64)
        assert np.all(np.isfinite(got))
        # O(1) outputs to the operator tolerance; the spike itself is sqrt(width) large: half an ulp of fp16 there
        small = np.abs(want) < 4.0
        gate(np.where(small, got, 0.0), np.where(small, want, 0.0), f"layernorm {name} {rows}x{width}", OP_MAX, OP_MEAN)
        rel = np.abs(got - want)[~small] / np.abs(want[~small]) if (~small).any() else np.zeros(1)
        assert rel.max() <= 2e-3, (name, rel.max())


@pytest.mark.parametrize("rows,width", [(5, 3072), (3, 49152), (4, 100), (2, 16392), (70000, 64)])
def test_bias_gelu_and_bias_residual(eet, rows, width):
    x = (wl.normal(111, width, (rows, width)).astype(np.float32) * 2.0).astype(np.float16)
    b = wl.normal(112, width, (width,), 0.5)
    r = wl.normal(113, width, (rows, width))
    y = torch.full((rows, width), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_bias_gelu(dev(x), dev(b), y)
    torch.cuda.synchronize()
    gate(host(y), orc.bias_gelu(x, b), f"bias_gelu {rows}x{width}", OP_MAX, OP_MEAN)
    y.fill_(float("nan"))
    eet.eet_op_bias_residual(dev(x), dev(b), dev(r), y)
    torch.cuda.synchronize()
    gate(host(y), orc.bias_residual(x, b, r), f"bias_residual {rows}x{width}", OP_MAX, OP_MEAN)


def test_gelu_at_the_ends_of_the_fp16_range(eet):
    """Arguments from the smallest to the largest fp16 magnitudes: exact limits (x for large x, -0 for very negative x),
    no NaN from an overflowing exponential, and the operator tolerance relative to the size of the value in between."""
    vals = [0.0, -0.0, 6e-8, -6e-8, 1e-4, -1e-4, 0.5, -0.5, 1.0, -1.0, 3.0, -3.0, 5.0, -5.0, 8.0, -8.0, 12.0, -12.0, 30.0, -30.0,
            100.0, -100.0, 1000.0, -1000.0, 30000.0, -30000.0, 65504.0, -65504.0]
    width = 64
    x = np.zeros((len(vals), width), np.float16)
    for r, v in enumerate(vals):
        x[r, :] = v
    b = np.zeros(width, np.float16)
    y = torch.full(x.shape, float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_bias_gelu(dev(x), dev(b), y)
    torch.cuda.synchronize()
    got = host(y).astype(np.float64)
    want = orc.gelu_tanh(x.astype(np.float64))
    assert np.all(np.isfinite(got))
    assert np.all(np.abs(got - want) <= np.maximum(2e-3, np.abs(want) * 2.0 ** -10)), np.abs(got - want).max(axis=1)
    for r, v in enumerate(vals):
        if v >= 12.0:
            assert np.all(got[r] == np.float64(np.float16(v)))          # gelu(x) = x to fp16 precision
        if v <= -12.0:
            assert np.all(got[r] == 0.0)


@pytest.mark.parametrize("B,nh,S,lens", [
    (3, 2, 9, [9, 1, 5]),              # scalar path (S % 8 != 0)
    (4, 1, 10, [5, 2, 4, 10]),         # the uneven batch of the paper's Section 4.1 example
    (2, 3, 64, [64, 17]),
    (2, 2, 520, [333, 520]),           # two vectors per lane, ragged
    (1, 2, 1024, [1000]),
    (2, 1, 4096, [4096, 2049]),        # the longest row the paper targets
    (1, 1, 4224, [4200]),
])
def test_softmax_maskfree(eet, B, nh, S, lens):
    s = wl.scores(200 + S, B, nh, S)
    # entries the method must never use: masked part of valid rows and whole pad rows get NaN
    poisoned = s.copy()
    iu = np.triu_indices(S, 1)
    poisoned[:, :, iu[0], iu[1]] = np.nan
    for b, L in enumerate(lens):
        poisoned[b, :, L:, :] = np.nan
    t = dev(poisoned)
    eet.eet_op_softmax_maskfree(t, lens, 0.37)
    torch.cuda.synchronize()
    got = host(t)
    want = orc.softmax_maskfree(s, lens, 0.37)
    for b, L in enumerate(lens):
        gate(got[b, :, :L], want[b, :, :L], f"softmax b={b}", 1e-3, 1e-4)
        assert np.all(got[b, :, :L][:, np.triu_indices(L, 1)[0], np.triu_indices(L, 1)[1]] == 0)
        assert np.all(got[b, :, :L, L:] == 0)                     # masked entries are exact zeros
        assert np.all(np.isnan(got[b, :, L:, :]))                 # pad rows untouched
        np.testing.assert_allclose(got[b, :, :L].astype(np.float64).sum(-1), 1.0, atol=4e-3)


@pytest.mark.parametrize("B,nh,S,lens", [
    (3, 2, 9, [9, 1, 5]),              # scalar path (S % 8 != 0)
    (4, 1, 10, [5, 2, 4, 10]),
    (2, 3, 64, [64, 17]),
    (2, 2, 520, [333, 520]),
    (2, 1, 4096, [4093, 2049]),        # windows that start and end inside 8-wide vectors
])
def test_softmax_maskfree_left_padded(eet, B, nh, S, lens):
    """Algorithm 1 in the layout it is printed for: pads first, rows padLen..S-1, window padLen..i."""
    s = wl.scores(230 + S, B, nh, S)
    poisoned = s.copy()
    iu = np.triu_indices(S, 1)
    poisoned[:, :, iu[0], iu[1]] = np.nan                         # keys after the query
    for b, L in enumerate(lens):
        poisoned[b, :, :S - L, :] = np.nan                        # rows of pad queries
        poisoned[b, :, :, :S - L] = np.nan                        # pad keys
    t = dev(poisoned)
    eet.eet_op_softmax_maskfree_left_padded(t, lens, 0.37)
    torch.cuda.synchronize()
    got = host(t)
    want = orc.softmax_maskfree(s, lens, 0.37, left_padded=True)
    for b, L in enumerate(lens):
        pad = S - L
        gate(got[b, :, pad:], want[b, :, pad:], f"left-padded softmax b={b}", 1e-3, 1e-4)
        assert np.all(got[b, :, pad:, :pad] == 0)                 # masked entries are exact zeros
        assert np.all(got[b, :, pad:][:, np.triu_indices(L, 1)[0], pad + np.triu_indices(L, 1)[1]] == 0)
        assert np.all(np.isnan(got[b, :, :pad, :]))               # pad rows untouched
        np.testing.assert_allclose(got[b, :, pad:].astype(np.float64).sum(-1), 1.0, atol=4e-3)


@pytest.mark.parametrize("M", [1, 5, 16, 17, 130, 200, 300, 513])
@pytest.mark.parametrize("K,N", [(64, 64), (128, 320), (256, 192), (1024, 3072), (4096, 1024), (1088, 1216), (1024, 2048), (4608, 3072), (512, 32832), (1280, 1280)])
def test_linear(eet, M, K, N):
    x = wl.normal(300 + M, K, (M, K))
    w = wl.normal(301, K * 7 + N, (N, K), 1.0 / np.sqrt(K))
    b = wl.normal(302, N, (N,), 0.5)
    r = wl.normal(303 + M, N, (M, N))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    xd, wd, bd, rd = dev(x), dev(w), dev(b), dev(r)
    lin = orc.linear(x, w, b)
    eet.eet_op_linear(xd, wd, bd, y)
    torch.cuda.synchronize()
    gate(host(y), lin, f"linear {M}x{K}x{N}", OP_MAX, OP_MEAN)
    y.fill_(float("nan"))
    eet.eet_op_linear(xd, wd, bd, y, act=1)
    torch.cuda.synchronize()
    gate(host(y), orc.gelu_tanh(lin), f"linear+gelu {M}x{K}x{N}", OP_MAX, OP_MEAN)
    y.fill_(float("nan"))
    eet.eet_op_linear(xd, wd, bd, y, residual=rd)
    torch.cuda.synchronize()
    gate(host(y), lin + r.astype(np.float64), f"linear+res {M}x{K}x{N}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("M,K,N", [(16, 512, 12288), (9, 256, 12288), (5, 768, 12288), (2, 256, 49152),   # 48 columns per workgroup
                                   (16, 512, 16384), (11, 256, 65536),                                     # 64 columns per workgroup
                                   (40, 256, 12288)])                                                      # the same in row slices
def test_linear_weight_stream_with_wide_workgroups(eet, M, K, N):
    """Decode-sized rows over outputs wide enough for the weight-streaming kernel to give a workgroup 48 or 64 columns."""
    x = wl.normal(370, M, (M, K))
    w = wl.normal(371, N, (N, K), 1.0 / np.sqrt(K))
    b = wl.normal(372, N, (N,), 0.5)
    r = wl.normal(373, M, (M, N))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    lin = orc.linear(x, w, b)
    eet.eet_op_linear(dev(x), dev(w), dev(b), y, act=1)
    torch.cuda.synchronize()
    gate(host(y), orc.gelu_tanh(lin), f"wide-workgroup stream linear+gelu {M}x{K}x{N}", OP_MAX, OP_MEAN)
    y.fill_(float("nan"))
    eet.eet_op_linear(dev(x), dev(w), dev(b), y, residual=dev(r))
    torch.cuda.synchronize()
    gate(host(y), lin + r.astype(np.float64), f"wide-workgroup stream linear+res {M}x{K}x{N}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("M,K,N", [(3000, 1024, 4160), (4099, 192, 3136), (2049, 4096, 6144)])
def test_linear_large_tiles(eet, M, K, N):
    """Shapes that take the 256x256 direct-to-LDS tile kernel, with ragged row and column tails."""
    x = wl.normal(350, M, (M, K))
    w = wl.normal(351, N, (N, K), 1.0 / np.sqrt(K))
    b = wl.normal(352, N, (N,), 0.5)
    r = wl.normal(353, M, (M, N))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    lin = orc.linear(x, w, b)
    eet.eet_op_linear(dev(x), dev(w), dev(b), y, act=1)
    torch.cuda.synchronize()
    gate(host(y), orc.gelu_tanh(lin), f"large linear+gelu {M}x{K}x{N}", OP_MAX, OP_MEAN)
    y.fill_(float("nan"))
    eet.eet_op_linear(dev(x), dev(w), dev(b), y, residual=dev(r))
    torch.cuda.synchronize()
    gate(host(y), lin + r.astype(np.float64), f"large linear+res {M}x{K}x{N}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("M,K,N,padx,pady", [(3000, 1024, 4160, 64, 72),     # 256x256 tiles, four waves
                                              (300, 512, 640, 8, 64),          # the small tiles
                                              (2049, 4096, 6144, 64, 0),
                                              (8492, 256, 4096, 64, 72),       # 544 large tiles: two whole rounds of 8192 rows, then 300 rows on small tiles
                                              (2648, 256, 16384, 64, 0)])      # 704 large tiles: two whole rounds of 2048 rows, then 600 rows on large tiles again
def test_linear_strided(eet, M, K, N, padx, pady):
    """eet_op_linear_strided: x and y are column slices of wider buffers (the layout the layer gives its feed-forward
    rows); the columns between the rows are neither read into the result nor written."""
    x = wl.normal(360, M, (M, K))
    w = wl.normal(361, N, (N, K), 1.0 / np.sqrt(K))
    b = wl.normal(362, N, (N,), 0.5)
    r = wl.normal(363, M, (M, N))
    xw = torch.full((M, K + padx), float("nan"), dtype=torch.float16, device="cuda:0")     # poison between the rows
    xw[:, :K] = dev(x)
    yw = torch.full((M, N + pady), float("nan"), dtype=torch.float16, device="cuda:0")
    lin = orc.linear(x, w, b)
    eet.eet_op_linear_strided(xw[:, :K], dev(w), dev(b), yw[:, :N], act=1)
    torch.cuda.synchronize()
    gate(host(yw[:, :N].contiguous()), orc.gelu_tanh(lin), f"strided linear+gelu {M}x{K}x{N}", OP_MAX, OP_MEAN)
    assert bool(torch.isnan(yw[:, N:]).all()), "columns between the output rows were written"
    yw.fill_(float("nan"))
    eet.eet_op_linear_strided(xw[:, :K], dev(w), dev(b), yw[:, :N], residual=dev(r))
    torch.cuda.synchronize()
    gate(host(yw[:, :N].contiguous()), lin + r.astype(np.float64), f"strided linear+res {M}x{K}x{N}", OP_MAX, OP_MEAN)
    assert bool(torch.isnan(yw[:, N:]).all())
    dense = torch.empty((M, N), dtype=torch.float16, device="cuda:0")                       # dense strides: the same call as eet_op_linear
    eet.eet_op_linear_strided(dev(x), dev(w), dev(b), dense, residual=dev(r))
    torch.cuda.synchronize()
    gate(host(dense), lin + r.astype(np.float64), f"linear+res through the strided entry point, dense rows {M}x{K}x{N}", OP_MAX, OP_MEAN)
    if M > 512:                                    # the same tile kernel serves both (few dense rows may go to row slices instead)
        assert np.array_equal(host(dense).view(np.uint16), host(yw[:, :N].contiguous()).view(np.uint16))


@pytest.mark.parametrize("M,K,N,what", [(8192, 128, 4096, "32 x 16 tiles in two rounds: one 16 x 16 super-block per round"),
                                        (6144, 64, 49152, "24 x 192 tiles in 18 rounds: eight blocks of one row group side by side")])
def test_linear_tile_orders_of_whole_rounds(eet, M, K, N, what):
    """Whole rounds of 256 x 256 tiles are handed to the XCDs in orders of their own: every output element is still written
    exactly once with the right value (sampled rows against the oracle, the first and last rows of tiles among them; the
    whole output finite, i.e. written)."""
    x = wl.normal(380, M, (M, K))
    w = wl.normal(381, N, (N, K), 1.0 / np.sqrt(K))
    b = wl.normal(382, N, (N,), 0.5)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_linear(dev(x), dev(w), dev(b), y)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all()), "some tile was not written"
    rng = np.random.default_rng(M + N)
    rows = sorted({0, 255, 256, 2047, 2048, 4095, 4096, M - 257, M - 256, M - 1} | {int(v) for v in rng.integers(0, M, 54)})
    want = orc.linear(x[rows], w, b)
    gate(host(y[rows]), want, f"linear {M}x{K}x{N} ({what})", OP_MAX, OP_MEAN)


def test_linear_strided_refuses_what_it_cannot_do(eet):
    K, N = 256, 512
    w, b = dev(wl.normal(364, 1, (N, K))), dev(wl.normal(365, 1, (N,)))
    xw = torch.zeros((8, K + 64), dtype=torch.float16, device="cuda:0")
    y = torch.empty((8, N), dtype=torch.float16, device="cuda:0")
    with pytest.raises(RuntimeError, match="weight-streaming"):          # 8 rows: the decode path, dense rows only
        eet.eet_op_linear_strided(xw[:, :K], w, b, y)
    eet.eet_op_linear_strided(xw[:, :K].contiguous(), w, b, y)           # dense: served
    L = eet.lib()
    assert L.eet_op_linear_strided(xw.data_ptr(), K - 8, w.data_ptr(), b.data_ptr(), None, y.data_ptr(), N, 300, K, N, 0, None) == -1
    assert L.eet_op_linear_strided(xw.data_ptr(), K + 4, w.data_ptr(), b.data_ptr(), None, y.data_ptr(), N, 300, K, N, 0, None) == -1
    torch.cuda.synchronize()


@pytest.mark.parametrize("d,heads,S,cap,lens", [
    (64, 2, 24, 32, [24, 1, 7]),
    (64, 3, 200, 224, [200, 3, 129, 64, 65]),
    (128, 2, 333, 352, [333, 40, 129]),
    (128, 1, 1030, 1030, [1030, 512]),
    (128, 2, 520, 544, [256, 257, 255, 512, 33, 1, 520, 289]),   # 256-row tiles: ends on, before and after tile and half-tile edges
    (64, 2, 520, 544, [256, 257, 129, 520]),
])
def test_attention_prefill(eet, d, heads, S, cap, lens):
    B, H = len(lens), heads * d
    q = wl.normal(400 + d, 1, (B, S, heads, d))
    k = wl.normal(400 + d, 2, (B, S, heads, d))
    v = wl.normal(400 + d, 3, (B, S, heads, d))
    want = orc.attention_prefill(q, k, v, lens)
    kc = np.full((B, heads, cap, d), np.nan, np.float16)          # slots >= L must never be read
    vc = np.full((B, heads, cap, d), np.nan, np.float16)
    qp = q.copy()
    for b, L in enumerate(lens):
        kc[b, :, :L] = k[b, :L].transpose(1, 0, 2)
        vc[b, :, :L] = v[b, :L].transpose(1, 0, 2)
        qp[b, L:] = np.nan                                        # pad queries must never be read
    ctx = torch.full((B, S, H), 7.0, dtype=torch.float16, device="cuda:0")
    eet.eet_op_attention_prefill(dev(qp.reshape(B, S, H)), dev(kc), dev(vc), ctx, lens, heads)
    torch.cuda.synchronize()
    got = host(ctx).reshape(B, S, heads, d)
    for b, L in enumerate(lens):
        gate(got[b, :L], want[b, :L], f"attention prefill b={b} L={L}", OP_MAX, OP_MEAN)
        assert np.all(got[b, L:] == 7.0)                          # pad rows are not written by the op


@pytest.mark.parametrize("d,heads,lens,causal", [
    (128, 40, [2048, 1024, 1025, 1791, 1793, 1536, 2047, 1280, 1777], True),      # 256-row kernel, 360 pairs in chunks of 48
    (128, 40, [2048, 1024, 1025, 1791, 1793, 1536, 2047, 1280, 1777], False),
    (64, 40, [2048, 1024, 1025, 1791, 1793, 1536, 2047, 1280, 1777, 2000, 1100, 1999, 1500, 1600, 1700, 1800, 1900, 1234, 1357, 1111], True),   # 128-row kernel, 800 pairs
])
def test_attention_prefill_in_chunks_of_pairs(eet, d, heads, lens, causal):
    """More K/V than the memory-side cache holds (285 and 330 MB): the launch takes the (sequence, head) pairs in chunks
    of 48, the last one ragged.  Sampled queries of every sequence, all heads, against the oracle; rows that no workgroup
    may write keep their fill."""
    S = 2048
    B, H = len(lens), heads * d
    assert sum(lens) * H * 4 > 256 << 20 and (B * heads) % 48 != 0
    q = wl.normal(431, 1, (B, S, heads, d))
    k = wl.normal(431, 2, (B, S, heads, d))
    v = wl.normal(431, 3, (B, S, heads, d))
    kc = torch.full((B, heads, S, d), float("nan"), dtype=torch.float16, device="cuda:0")
    vc = torch.full((B, heads, S, d), float("nan"), dtype=torch.float16, device="cuda:0")
    for b, L in enumerate(lens):
        kc[b, :, :L] = dev(k[b, :L]).permute(1, 0, 2)
        vc[b, :, :L] = dev(v[b, :L]).permute(1, 0, 2)
    ctx = torch.full((B, S, H), 7.0, dtype=torch.float16, device="cuda:0")
    op = eet.eet_op_attention_prefill if causal else eet.eet_op_attention_encoder
    op(dev(q.reshape(B, S, H)), kc, vc, ctx, lens, heads)
    torch.cuda.synchronize()
    rng = np.random.default_rng(432)
    for b, L in enumerate(lens):
        assert bool((ctx[b, L:] == 7.0).all())                    # pad rows are not written by the op
        Kb = np.ascontiguousarray(np.asarray(k[b, :L], np.float64).transpose(1, 0, 2))
        Vb = np.ascontiguousarray(np.asarray(v[b, :L], np.float64).transpose(1, 0, 2))
        rows = sorted({0, 255, 256, L - 257, L - 1} | {int(t) for t in rng.integers(0, L, 4)})
        want = np.stack([orc.attend(np.asarray(q[b, t], np.float64), Kb, Vb, t + 1 if causal else L) for t in rows])
        got = host(ctx[b, rows]).reshape(len(rows), heads, d)
        gate(got, want, f"attention prefill in chunks b={b} L={L} causal={causal}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("d,heads,S,cap,lens", [
    (128, 2, 1100, 1104, [1100, 700]),        # 256-row kernel
    (128, 2, 500, 512, [500, 257]),           # 128-row kernel, heads of 128
    (64, 2, 700, 704, [700, 130]),            # 128-row kernel, heads of 64
])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_prefill_with_a_wide_score_range_and_a_rising_maximum(eet, d, heads, S, cap, lens, causal):
    """Scores with a standard deviation of about 12 whose magnitude grows with the key position: the running maximum
    keeps rising from key tile to key tile by more than the slack the kernels allow before they move the reference of
    their exponentials, so the rescaling path runs many times per row, and the softmax is close to one-hot."""
    B, H = len(lens), heads * d
    q = (wl.normal(430 + d, 1, (B, S, heads, d)).astype(np.float32) * 4.0).astype(np.float16)
    ramp = (1.0 + 2.0 * np.arange(S, dtype=np.float32) / S)[None, :, None, None]
    k = (wl.normal(430 + d, 2, (B, S, heads, d)).astype(np.float32) * ramp).astype(np.float16)
    v = wl.normal(430 + d, 3, (B, S, heads, d))
    want = orc.attention_prefill(q, k, v, lens, causal=causal)
    kc = np.full((B, heads, cap, d), np.nan, np.float16)
    vc = np.full((B, heads, cap, d), np.nan, np.float16)
    for b, L in enumerate(lens):
        kc[b, :, :L] = k[b, :L].transpose(1, 0, 2)
        vc[b, :, :L] = v[b, :L].transpose(1, 0, 2)
    ctx = torch.zeros((B, S, H), dtype=torch.float16, device="cuda:0")
    op = eet.eet_op_attention_prefill if causal else eet.eet_op_attention_encoder
    op(dev(q.reshape(B, S, H)), dev(kc), dev(vc), ctx, lens, heads)
    nk = torch.tensor(lens, dtype=torch.int32, device="cuda:0")
    last_q = np.stack([q[b, L - 1] for b, L in enumerate(lens)]).reshape(B, H)
    dctx = torch.zeros((B, H), dtype=torch.float16, device="cuda:0")
    scratch = torch.empty(eet.eet_op_attention_decode_scratch_bytes(B, heads, d, cap), dtype=torch.uint8, device="cuda:0")
    eet.eet_op_attention_decode(dev(last_q), dev(kc), dev(vc), dctx, nk, scratch)      # the last row again, as a decode step
    torch.cuda.synchronize()
    got = host(ctx).reshape(B, S, heads, d)
    for b, L in enumerate(lens):
        gate(got[b, :L], want[b, :L], f"wide-range attention (causal={causal}) b={b} L={L}", OP_MAX, OP_MEAN)
        gate(host(dctx)[b].reshape(heads, d), want[b, L - 1], f"wide-range attention decode b={b}", OP_MAX, OP_MEAN)   # the last row sees all keys either way


@pytest.mark.parametrize("d,heads,S,cap,lens", [
    (64, 2, 24, 32, [24, 1, 7]),
    (64, 3, 200, 224, [200, 3, 129, 64, 65]),
    (128, 2, 333, 352, [333, 40, 129, 128]),
    (128, 1, 1030, 1030, [1030, 512]),
    (128, 2, 520, 544, [256, 257, 255, 512, 33, 1, 520, 289]),
    (64, 2, 520, 544, [256, 257, 129, 520]),
])
def test_attention_encoder(eet, d, heads, S, cap, lens):
    """Padding skip only, no sequence mask: every valid row sees all valid keys of its sequence."""
    B, H = len(lens), heads * d
    q = wl.normal(450 + d, 1, (B, S, heads, d))
    k = wl.normal(450 + d, 2, (B, S, heads, d))
    v = wl.normal(450 + d, 3, (B, S, heads, d))
    want = orc.attention_prefill(q, k, v, lens, causal=False)
    kc = np.full((B, heads, cap, d), np.nan, np.float16)          # slots >= L must never be read
    vc = np.full((B, heads, cap, d), np.nan, np.float16)
    qp = q.copy()
    for b, L in enumerate(lens):
        kc[b, :, :L] = k[b, :L].transpose(1, 0, 2)
        vc[b, :, :L] = v[b, :L].transpose(1, 0, 2)
        qp[b, L:] = np.nan                                        # pad queries must never be read
    ctx = torch.full((B, S, H), 7.0, dtype=torch.float16, device="cuda:0")
    eet.eet_op_attention_encoder(dev(qp.reshape(B, S, H)), dev(kc), dev(vc), ctx, lens, heads)
    torch.cuda.synchronize()
    got = host(ctx).reshape(B, S, heads, d)
    for b, L in enumerate(lens):
        gate(got[b, :L], want[b, :L], f"attention encoder b={b} L={L}", OP_MAX, OP_MEAN)
        assert np.all(got[b, L:] == 7.0)                          # pad rows are not written by the op


@pytest.mark.parametrize("d,heads,S,cap,lens", [
    (64, 2, 24, 32, [24, 1, 7]),
    (64, 3, 200, 224, [200, 3, 129, 64, 65]),
    (128, 2, 336, 352, [333, 40, 129, 128]),
    (128, 1, 520, 520, [520, 256, 257]),
])
def test_attention_unfused(eet, d, heads, S, cap, lens):
    """Paper-form attention: materialised scores from the buffer manager, Algorithm 1 in place, then P.V.
    Tolerance: the raw scores pass through fp16 before the exponent, so a probability carries a relative error of
    up to max|s| * 2^-11 / sqrt(d) on top of its own rounding; the context inherits it (bound written below)."""
    B, H = len(lens), heads * d
    q = wl.normal(470 + d, 1, (B, S, heads, d))
    k = wl.normal(470 + d, 2, (B, S, heads, d))
    v = wl.normal(470 + d, 3, (B, S, heads, d))
    want = orc.attention_prefill(q, k, v, lens)
    raw = np.einsum("bihd,bjhd->bhij", q.astype(np.float64), k.astype(np.float64))
    want_p = orc.softmax_maskfree(raw, lens, 1.0 / np.sqrt(d))
    kc = np.full((B, heads, cap, d), np.nan, np.float16)          # slots >= L must never be read
    vc = np.full((B, heads, cap, d), np.nan, np.float16)
    qp = q.copy()
    for b, L in enumerate(lens):
        kc[b, :, :L] = k[b, :L].transpose(1, 0, 2)
        vc[b, :, :L] = v[b, :L].transpose(1, 0, 2)
        qp[b, L:] = np.nan                                        # pad queries must never be read
    score_bytes = B * heads * S * S * 2
    arena = torch.full((score_bytes + 4096,), 0x7E, dtype=torch.uint8, device="cuda:0")     # 0x7E7E is a NaN pattern in fp16
    base = (arena.data_ptr() + 255) // 256 * 256
    mgr = eet.eet_bufmgr_create(base, score_bytes + 256)
    ctx = torch.full((B, S, H), 7.0, dtype=torch.float16, device="cuda:0")
    rel = float(max(np.abs(raw[b, :, :L, :L]).max() for b, L in enumerate(lens))) * 2.0 ** -11 / np.sqrt(d)
    for call in range(2):                                          # the second call reuses the idle score buffer
        eet.eet_op_attention_unfused(dev(qp.reshape(B, S, H)), dev(kc), dev(vc), ctx, lens, heads, mgr, module=0)
        torch.cuda.synchronize()
        got = host(ctx).reshape(B, S, heads, d)
        for b, L in enumerate(lens):
            gate(got[b, :L], want[b, :L], f"unfused attention b={b} L={L} call {call}",
                 OP_MAX + rel * float(np.abs(v[b, :L]).max()), OP_MEAN + rel)
            assert np.all(got[b, L:] == 7.0)                      # pad rows are not written by the op
    st = eet.eet_bufmgr_query(mgr)
    assert (st.created, st.reused_same_size, st.idle, st.footprint_bytes) == (1, 1, 1, (score_bytes + 255) // 256 * 256)
    # the probabilities Algorithm 1 left in the buffer: request it again (same module, same size: the same buffer)
    ptr = eet.eet_bufmgr_request(mgr, score_bytes, 0)
    assert ptr == base
    off = base - arena.data_ptr()
    probs = arena[off:off + score_bytes].view(torch.float16).reshape(B, heads, S, S).cpu().numpy().astype(np.float64)
    for b, L in enumerate(lens):
        assert np.abs(probs[b, :, :L, :] - want_p[b, :, :L, :]).max() <= 1e-3 + rel        # zeros right of the diagonal included
    eet.eet_bufmgr_release(mgr, ptr)
    eet.eet_bufmgr_destroy(mgr)


@pytest.mark.parametrize("d,heads,cap,n_keys", [
    (64, 16, 640, [640, 1, 63, 64, 65, 300, 511, 129]),     # 128 (sequence, head) pairs: one key range each, no merge launch
    (128, 32, 520, [520, 257, 32, 33]),
])
@pytest.mark.parametrize("peaked", [False, True])
def test_attention_decode_with_one_range_per_pair(eet, d, heads, cap, n_keys, peaked):
    B = len(n_keys)
    q = wl.normal(520 + d, 1, (B, heads, d))
    kc = wl.normal(520 + d, 2, (B, heads, cap, d))
    vc = wl.normal(520 + d, 3, (B, heads, cap, d))
    if peaked:        # scores with a standard deviation of about 12 that grow with the slot: the running maximum keeps moving
        q = (q.astype(np.float32) * 4.0).astype(np.float16)
        kc = (kc.astype(np.float32) * (1.0 + 2.0 * np.arange(cap, dtype=np.float32) / cap)[None, None, :, None]).astype(np.float16)
    assert eet.eet_op_attention_decode_scratch_bytes(B, heads, d, cap) <= 256      # nothing to merge
    want = orc.attention_decode(q, kc, vc, n_keys)
    kp, vp = kc.copy(), vc.copy()
    for b, n in enumerate(n_keys):
        kp[b, :, n:] = np.nan
        vp[b, :, n:] = np.nan
    scratch = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    ctx = torch.full((B, heads * d), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_attention_decode(dev(q.reshape(B, heads * d)), dev(kp), dev(vp), ctx, dev(np.asarray(n_keys, np.int32)), scratch)
    torch.cuda.synchronize()
    gate(host(ctx).reshape(B, heads, d), want, f"attention decode, one range, d={d} peaked={peaked}", OP_MAX, OP_MEAN)


@pytest.mark.parametrize("d,heads,cap,n_keys", [
    (64, 64, 256, [0, 5, 0]),           # 192 pairs: one key range per pair
    (128, 2, 4224, [0, 4224, -3]),      # few pairs: the key range is split and merged by the combine kernel
])
def test_attention_decode_of_a_sequence_without_keys_is_zero(eet, d, heads, cap, n_keys):
    """n_keys[b] < 1 lives on the device and cannot be refused by the host: the context rows of such a sequence are
    defined as zeros (not NaN), the other sequences do not notice."""
    B = len(n_keys)
    q = wl.normal(520 + d, 1, (B, heads, d))
    kc = wl.normal(520 + d, 2, (B, heads, cap, d))
    vc = wl.normal(520 + d, 3, (B, heads, cap, d))
    seen = [max(n, 0) for n in n_keys]
    live = [b for b in range(B) if seen[b] > 0]
    want = orc.attention_decode(q[live], kc[live], vc[live], [seen[b] for b in live])
    scratch = torch.empty(eet.eet_op_attention_decode_scratch_bytes(B, heads, d, cap), dtype=torch.uint8, device="cuda:0")
    scratch.fill_(0xFF)                                   # NaN patterns where partial results will land
    ctx = torch.full((B, heads * d), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_attention_decode(dev(q.reshape(B, heads * d)), dev(kc), dev(vc), ctx, dev(np.asarray(n_keys, np.int32)), scratch)
    torch.cuda.synchronize()
    got = host(ctx).reshape(B, heads, d)
    for i, b in enumerate(live):
        gate(got[b], want[i], f"attention decode beside sequences without keys, d={d} b={b}", OP_MAX, OP_MEAN)
    for b in range(B):
        if seen[b] == 0:
            assert np.all(got[b] == 0), f"sequence {b} has no key: its context must be zeros"


@pytest.mark.parametrize("d,heads,cap,n_keys", [
    (64, 4, 600, [1, 17, 600]),
    (128, 4, 600, [600, 16, 33]),
    (64, 2, 2048, [2048, 100]),        # several key ranges per (sequence, head), one of them empty for the short one
    (128, 2, 4224, [4224, 1]),
])
def test_attention_decode(eet, d, heads, cap, n_keys):
    B = len(n_keys)
    q = wl.normal(500 + d, 1, (B, heads, d))
    kc = wl.normal(500 + d, 2, (B, heads, cap, d))
    vc = wl.normal(500 + d, 3, (B, heads, cap, d))
    want = orc.attention_decode(q, kc, vc, n_keys)
    kp, vp = kc.copy(), vc.copy()
    for b, n in enumerate(n_keys):
        kp[b, :, n:] = np.nan
        vp[b, :, n:] = np.nan
    scratch = torch.empty(eet.eet_op_attention_decode_scratch_bytes(B, heads, d, cap), dtype=torch.uint8, device="cuda:0")
    ctx = torch.full((B, heads * d), float("nan"), dtype=torch.float16, device="cuda:0")
    qd, kd, vd, nd = dev(q.reshape(B, heads * d)), dev(kp), dev(vp), dev(np.asarray(n_keys, np.int32))
    first = None
    for rep in range(2):          # the scratch is reused as it is
        ctx.fill_(float("nan"))
        eet.eet_op_attention_decode(qd, kd, vd, ctx, nd, scratch)
        torch.cuda.synchronize()
        gate(host(ctx).reshape(B, heads, d), want, f"attention decode d={d} call {rep}", OP_MAX, OP_MEAN)
        if first is None:
            first = host(ctx).copy()
        assert np.array_equal(first.view(np.uint16), host(ctx).view(np.uint16))      # bitwise reproducible
