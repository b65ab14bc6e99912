"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself
(brute force with explicit masks, invariants, closed forms, torch float64 on the unpadded
special case, and the integers the paper prints).  CPU only."""
import math
import os
import re

import numpy as np
import pytest

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl
from tests import bruteforce as bf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = [t.strip() for t in line.split("=", 1)]
            out[k] = v
    return out


def tiny_weights(seed, H, F, sigma=0.3, affine=True):
    w = wl.Workload("t", seed, H, 1, F, 1, 1, 1, 1, 1, 0, 1, sigma_w=sigma)
    W = wl.layer_weights(w, random_affine=affine)
    return {k: v.astype(np.float64) for k, v in W.items()}


def make_layer(W, heads, B, max_seq):
    return orc.DecoderLayerOracle(W, heads, B, max_seq)


# ------------------------------------------------------------------ brute force, explicit masks
@pytest.mark.parametrize("lens,S,H,heads,F", [
    ([7, 4, 1], 7, 16, 2, 32),
    ([5, 2, 4, 10], 10, 8, 2, 16),      # the uneven batch the paper uses as its example
    ([3, 6], 6, 12, 3, 24),
])
def test_layer_matches_additive_mask_bruteforce(lens, S, H, heads, F):
    g = golden()
    if lens == [5, 2, 4, 10]:
        assert [int(t) for t in g["ragged_batch_example"].split(",")] == lens
        assert int(g["ragged_batch_prefill_len"]) == S == max(lens)
    W = tiny_weights(3, H, F)
    x = wl.normal(5, 1, (len(lens), S, H)).astype(np.float64)
    got = make_layer(W, heads, len(lens), S).prefill(x, lens)
    want = bf.masked_layer(x, lens, W, heads)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(got[b, :L], want[b, :L], rtol=0, atol=1e-9)
        assert np.all(got[b, L:] == 0.0)


def test_softmax_op_matches_additive_mask_bruteforce():
    lens = [9, 1, 5]
    s = wl.scores(21, 3, 2, 9).astype(np.float64)
    got = orc.softmax_maskfree(s, lens, scale=0.7)
    want = bf.masked_softmax(s, lens, scale=0.7)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    for b, L in enumerate(lens):
        assert np.array_equal(got[b, :, L:], s[b, :, L:])            # pad rows untouched
        assert np.all(np.triu(got[b, 0, :L], 1) == 0.0)               # masked entries are zero
        np.testing.assert_allclose(got[b, :, :L].sum(-1), 1.0, atol=1e-12)


# ------------------------------------------------------------------ invariants the paper states
def test_causality_rows_unchanged_by_later_tokens():
    W = tiny_weights(4, 32, 64)
    lens = [11, 6]
    x = wl.normal(6, 1, (2, 12, 32)).astype(np.float64)
    base = make_layer(W, 4, 2, 12).prefill(x, lens)
    t = 4
    x2 = x.copy()
    x2[:, t + 1:] = wl.normal(6, 2, x2[:, t + 1:].shape).astype(np.float64) * 50.0
    pert = make_layer(W, 4, 2, 12).prefill(x2, lens)
    assert np.array_equal(base[:, : t + 1], pert[:, : t + 1])          # bitwise
    assert not np.allclose(base[0, t + 1: lens[0]], pert[0, t + 1: lens[0]])


@pytest.mark.parametrize("poison", [np.nan, np.inf, 1e4])
def test_valid_rows_independent_of_pad_content(poison):
    W = tiny_weights(8, 32, 64)
    lens = [3, 9, 1]
    x = wl.normal(9, 1, (3, 9, 32)).astype(np.float64)
    base = make_layer(W, 2, 3, 9).prefill(x, lens)
    x2 = x.copy()
    for b, L in enumerate(lens):
        x2[b, L:] = poison
    lay = make_layer(W, 2, 3, 9)
    pert = lay.prefill(x2, lens)
    assert np.array_equal(base, pert)                                   # skipped, not masked
    assert np.all(np.isfinite(pert))
    for b, L in enumerate(lens):                                        # pads never reach the cache
        assert np.all(np.isnan(lay.k_cache[b, :, L:])) and np.all(np.isfinite(lay.k_cache[b, :, :L]))


def test_decode_equals_prefill_of_extended_prompt():
    H, heads, F, S, steps = 24, 3, 48, 7, 4
    W = tiny_weights(10, H, F)
    lens = np.array([7, 2, 5])
    full = wl.normal(12, 1, (3, S + steps, H)).astype(np.float64)
    lay = make_layer(W, heads, 3, S + steps)
    lay.prefill(full[:, :S], lens)
    cur = lens.copy()
    for k in range(steps):
        xk = np.stack([full[b, cur[b]] for b in range(3)])
        got = lay.decode_step(xk)
        assert np.array_equal(lay.slot_log[-1], cur)                    # slot written = old n_b
        cur = cur + 1
        assert np.array_equal(lay.lens[:3], cur)
        ref = make_layer(W, heads, 3, S + steps).prefill(full, cur)
        for b in range(3):
            np.testing.assert_allclose(got[b], ref[b, cur[b] - 1], rtol=0, atol=1e-10)
    o = orc.padding_offsets(lens, S)
    assert o["pad_len"].tolist() == [0, 5, 2] and o["cu_seqlens"].tolist() == [0, 7, 9, 14]


# ------------------------------------------------------------------ closed forms
def test_first_row_context_is_v0_and_equal_keys_give_running_mean():
    heads, d, n = 2, 4, 6
    rng_v = wl.normal(30, 1, (heads, n, d)).astype(np.float64)
    q = wl.normal(30, 2, (heads, d)).astype(np.float64)
    K = wl.normal(30, 3, (heads, n, d)).astype(np.float64)
    np.testing.assert_array_equal(orc.attend(q, K, rng_v, 1), rng_v[:, 0])
    Keq = np.repeat(K[:, :1], n, axis=1)
    for i in range(n):
        np.testing.assert_allclose(orc.attend(q, Keq, rng_v, i + 1), rng_v[:, : i + 1].mean(1), atol=1e-13)


def test_scale_is_one_over_sqrt_d():
    # two keys, scores differ by exactly sqrt(d)*ln(3) before scaling -> weights 3/4, 1/4
    d = 16
    q = np.zeros((1, d)); q[0, 0] = 1.0
    K = np.zeros((1, 2, d)); K[0, 0, 0] = math.sqrt(d) * math.log(3.0)
    V = np.zeros((1, 2, d)); V[0, 0, 0] = 1.0; V[0, 1, 1] = 1.0
    o = orc.attend(q, K, V, 2)
    np.testing.assert_allclose(o[0, :2], [0.75, 0.25], atol=1e-13)


def test_zero_linear_weights_make_the_layer_the_identity():
    H, F = 16, 32
    W = tiny_weights(2, H, F)
    for k in ("w_qkv", "b_qkv", "w_o", "b_o", "w_fc1", "b_fc1", "w_fc2", "b_fc2"):
        W[k] = np.zeros_like(W[k])
    x = wl.normal(2, 9, (2, 5, H)).astype(np.float64)
    out = make_layer(W, 2, 2, 5).prefill(x, [5, 3])
    assert np.array_equal(out[0], x[0]) and np.array_equal(out[1, :3], x[1, :3])


def test_layernorm_statistics_and_affine():
    x = wl.normal(40, 1, (5, 1280)).astype(np.float64) * 3 + 2
    y = orc.layernorm(x, np.ones(1280), np.zeros(1280), 1e-5)
    var = x.var(axis=-1)                                               # numpy: biased by default
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose(y.var(-1), var / (var + 1e-5), rtol=1e-12)
    g = np.linspace(0.5, 1.5, 1280); b = np.linspace(-1, 1, 1280)
    np.testing.assert_allclose(orc.layernorm(x, g, b, 1e-5), y * g + b, atol=1e-13)
    # a constant row has zero deviation: output is beta exactly, eps keeps it finite
    np.testing.assert_array_equal(orc.layernorm(np.full((1, 8), 3.0), np.ones(8), b[:8], 1e-5)[0], b[:8])


def test_gelu_identities():
    x = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(orc.gelu_tanh(x) - orc.gelu_tanh(-x), x, atol=1e-14)
    assert orc.gelu_tanh(np.array([0.0]))[0] == 0.0
    # tanh form stays within 1e-3 of x*Phi(x) but is not equal to it
    exact = x * 0.5 * (1 + np.vectorize(math.erf)(x / math.sqrt(2)))
    diff = np.abs(orc.gelu_tanh(x) - exact).max()
    assert 1e-5 < diff < 1e-3
    np.testing.assert_allclose(orc.gelu_tanh(np.array([1.0]))[0], 0.8411919906082768, atol=1e-15)
    np.testing.assert_allclose(orc.bias_gelu(x, 0.5), orc.gelu_tanh(x + 0.5))
    np.testing.assert_array_equal(orc.bias_residual(np.array([1.0, 2.0]), np.array([0.5, 0.25]), np.array([4.0, 8.0])),
                                  [5.5, 10.25])


# ------------------------------------------------------------------ library special case
def test_unpadded_case_matches_torch_float64():
    torch = pytest.importorskip("torch")
    Fn = torch.nn.functional
    B, S, H, heads, F = 2, 33, 64, 4, 128
    d = H // heads
    W = tiny_weights(50, H, F, sigma=0.1)
    x = wl.normal(51, 1, (B, S, H)).astype(np.float64)
    got = make_layer(W, heads, B, S).prefill(x, [S] * B)
    T = {k: torch.from_numpy(v) for k, v in W.items()}
    xt = torch.from_numpy(x)
    a = Fn.layer_norm(xt, (H,), T["ln1_g"], T["ln1_b"], 1e-5)
    qkv = Fn.linear(a, T["w_qkv"], T["b_qkv"]).view(B, S, 3, heads, d).permute(2, 0, 3, 1, 4)
    ctx = Fn.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=True)
    y = xt + Fn.linear(ctx.transpose(1, 2).reshape(B, S, H), T["w_o"], T["b_o"])
    c = Fn.layer_norm(y, (H,), T["ln2_g"], T["ln2_b"], 1e-5)
    z = y + Fn.linear(Fn.gelu(Fn.linear(c, T["w_fc1"], T["b_fc1"]), approximate="tanh"), T["w_fc2"], T["b_fc2"])
    np.testing.assert_allclose(got, z.numpy(), rtol=0, atol=1e-10)
    # op-level attention against the same routine
    q4 = qkv[0].permute(0, 2, 1, 3).numpy(); k4 = qkv[1].permute(0, 2, 1, 3).numpy(); v4 = qkv[2].permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(orc.attention_prefill(q4, k4, v4, [S] * B),
                               ctx.permute(0, 2, 1, 3).numpy(), atol=1e-12)
    last = orc.attention_decode(q4[:, -1], k4.transpose(0, 2, 1, 3), v4.transpose(0, 2, 1, 3), [S] * B)
    np.testing.assert_allclose(last, ctx[:, :, -1].numpy(), atol=1e-12)


def test_sampled_rows_equal_full_evaluation():
    W = tiny_weights(60, 32, 64)
    x = wl.normal(61, 1, (3, 10, 32)).astype(np.float64)
    lens = [10, 4, 7]
    full = make_layer(W, 2, 3, 10).prefill(x, lens)
    part = make_layer(W, 2, 3, 10).prefill(x, lens, rows={0: [0, 9, 3], 2: [6]})
    for b, i in [(0, 0), (0, 9), (0, 3), (2, 6)]:
        np.testing.assert_allclose(full[b, i], part[b, i], rtol=0, atol=1e-12)   # matmul blocking differs
    assert np.all(np.isnan(part[1, :4])) and np.all(np.isnan(part[0, 1])) and np.all(part[1, 4:] == 0)


# ------------------------------------------------------------------ integers the paper prints
def test_fold_shape_follows_the_worked_example():
    g = golden()
    limit = int(g["fold_block_limit"])
    assert orc.fold_shape(int(g["fold_example_width"]), limit) == (int(g["fold_example_pieces"]), int(g["fold_example_threads"]))
    assert orc.fold_shape(1024, limit) == (1, 1024) and orc.fold_shape(768, limit) == (1, 768)
    for w in range(limit + 1, int(g["fold_max_hidden"]) + 1, 8):
        t, n = orc.fold_shape(w, limit)
        assert t & (t - 1) == 0 and t * n >= w and n <= limit
        assert n >= int(g["fold_min_threads_when_folded"])              # "minimum thread number is 512"
    assert orc.fold_shape(int(g["fold_max_hidden"]), limit) == (16, 1024)
    assert orc.fold_shape(int(g["fold_max_seq"]), limit) == (4, 1024)
    # the printed closed form does not reproduce the worked example: t = 2^(ceil(h/1024)-1), n = h/2^t
    h = int(g["fold_example_width"])
    t_printed = 2 ** (math.ceil(h / limit) - 1)
    assert h / 2 ** t_printed != int(g["fold_example_threads"])


def test_size_formulas():
    g = golden()
    b, h, s, l, p, n = 16, 1024, 1024, 24, 512, 16
    env = dict(b=b, h=h, s=s, l=l, p=p, n=n)
    assert re.fullmatch(r"[0-9a-z*+() ]+", g["kv_cache_formula"] + g["activation_cache_formula"] + g["buffer_formula"])
    assert orc.kv_cache_elements(b, h, s, l) == eval(g["kv_cache_formula"], {}, env)
    assert orc.activation_cache_elements(b, h, p) == eval(g["activation_cache_formula"], {}, env)
    assert orc.buffer_elements(b, p, h, n) == eval(g["buffer_formula"], {}, env)


# ------------------------------------------------------------------ encoder use (no sequence mask)
@pytest.mark.parametrize("lens,S,H,heads,F", [([7, 4, 1], 7, 16, 2, 32), ([3, 6], 6, 12, 3, 24)])
def test_encoder_matches_padding_mask_bruteforce(lens, S, H, heads, F):
    W = tiny_weights(3, H, F)
    x = wl.normal(5, 1, (len(lens), S, H)).astype(np.float64)
    got = make_layer(W, heads, len(lens), S).encode(x, lens)
    want = bf.masked_layer(x, lens, W, heads, causal_mask=False)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(got[b, :L], want[b, :L], rtol=0, atol=1e-9)
        assert np.all(got[b, L:] == 0.0)
    # and it is not the causal layer (except for one-token sequences and every last row)
    causal = make_layer(W, heads, len(lens), S).prefill(x, lens)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(got[b, L - 1], causal[b, L - 1], rtol=0, atol=1e-12)
        if L > 1:
            assert np.abs(got[b, 0] - causal[b, 0]).max() > 1e-6


def test_encoder_is_permutation_equivariant_and_pad_independent():
    """Without a sequence mask and without positions, permuting the valid tokens of a sequence
    permutes its outputs; pad content (NaN here) never matters."""
    W = tiny_weights(70, 32, 64)
    lens = [9, 5]
    x = wl.normal(71, 1, (2, 12, 32)).astype(np.float64)
    base = make_layer(W, 4, 2, 12).encode(x, lens)
    perm = np.array([4, 0, 8, 2, 6, 1, 7, 3, 5])
    xp = x.copy()
    xp[0, :9] = x[0, perm]
    xp[0, 9:] = np.nan
    xp[1, 5:] = np.nan
    got = make_layer(W, 4, 2, 12).encode(xp, lens)
    np.testing.assert_allclose(got[0, :9], base[0, perm], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(got[1, :5], base[1, :5])
    assert np.all(got[0, 9:] == 0) and np.all(got[1, 5:] == 0)


def test_encoder_unpadded_case_matches_torch_float64():
    torch = pytest.importorskip("torch")
    Fn = torch.nn.functional
    B, S, heads, d = 2, 21, 3, 8
    q = wl.normal(80, 1, (B, S, heads, d)).astype(np.float64)
    k = wl.normal(80, 2, (B, S, heads, d)).astype(np.float64)
    v = wl.normal(80, 3, (B, S, heads, d)).astype(np.float64)
    t = [torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v)]
    want = Fn.scaled_dot_product_attention(t[0], t[1], t[2], is_causal=False).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(orc.attention_prefill(q, k, v, [S] * B, causal=False), want, atol=1e-12)
    # shorter valid lengths = the library routine on the truncated sequence
    L = 13
    want_L = Fn.scaled_dot_product_attention(t[0][:, :, :L], t[1][:, :, :L], t[2][:, :, :L]).permute(0, 2, 1, 3).numpy()
    got_L = orc.attention_prefill(q, k, v, [L] * B, causal=False)
    np.testing.assert_allclose(got_L[:, :L], want_L, atol=1e-12)
    assert np.all(got_L[:, L:] == 0)


# ------------------------------------------------------------------ planted mistakes must be caught
class _Mutant:
    """Temporarily replace an attribute of the oracle module."""

    def __init__(self, name, fn):
        self.name, self.fn = name, fn

    def __enter__(self):
        self.old = getattr(orc, self.name)
        setattr(orc, self.name, self.fn)

    def __exit__(self, *a):
        setattr(orc, self.name, self.old)


def _attend_no_diag(q, K, V, n):      # window excludes the diagonal
    return _REAL["attend"](q, K, V, max(n - 1, 1))


def _attend_no_scale(q, K, V, n):     # forgets 1/sqrt(d)
    return _REAL["attend"](q * math.sqrt(q.shape[1]), K, V, n)


def _ln_unbiased(x, g, b, eps=1e-5):  # n-1 in the variance
    x = np.asarray(x, np.float64)
    mu = x.mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(x.var(-1, ddof=1, keepdims=True) + eps) * g + b


def _gelu_erf(x):
    return x * 0.5 * (1 + np.vectorize(math.erf)(x / math.sqrt(2)))


def _linear_transposed(x, w, b):      # uses W instead of W^T where the matrix is square
    w = np.asarray(w)
    return x @ (w if w.shape[0] == w.shape[1] else w.T) + b


_REAL = {"attend": orc.attend}


@pytest.mark.parametrize("name,fn", [("attend", _attend_no_diag), ("attend", _attend_no_scale),
                                     ("layernorm", _ln_unbiased), ("gelu_tanh", _gelu_erf),
                                     ("linear", _linear_transposed)])
def test_planted_mistakes_fail_the_bruteforce_pin(name, fn):
    with _Mutant(name, fn):
        with pytest.raises(AssertionError):
            test_layer_matches_additive_mask_bruteforce([7, 4, 1], 7, 16, 2, 32)


def _attend_causal_in_encoder(q, K, V, n):   # an encoder that still applies a sequence mask
    return _REAL["attend"](q, K, V, max(1, n - 1))


@pytest.mark.parametrize("name,fn", [("attend", _attend_causal_in_encoder), ("attend", _attend_no_scale)])
def test_planted_mistakes_fail_the_encoder_pin(name, fn):
    with _Mutant(name, fn):
        with pytest.raises(AssertionError):
            test_encoder_matches_padding_mask_bruteforce([7, 4, 1], 7, 16, 2, 32)


# ------------------------------------------------------------------ left-padded layout (the layout Algorithm 1 is printed for)
def shift_left(x, lens):
    """Right-padded [B, S, ...] -> left-padded: the valid rows of sequence b move to [S-L_b, S); pads are NaN."""
    out = np.full_like(np.asarray(x, np.float64), np.nan)
    S = x.shape[1]
    for b, L in enumerate(lens):
        out[b, S - L:] = x[b, :L]
    return out


@pytest.mark.parametrize("lens,S,H,heads,F", [([7, 4, 1], 7, 16, 2, 32), ([5, 2, 4, 10], 10, 8, 2, 16)])
def test_left_padded_layer_matches_additive_mask_bruteforce(lens, S, H, heads, F):
    """Algorithm 1 walks rows padLen .. seqLen-1 of a sequence and lets row i see keys padLen .. i: in that layout
    the oracle must equal dense scores + additive causal mask + additive mask on the leading pad columns."""
    W = tiny_weights(3, H, F)
    xr = wl.normal(5, 1, (len(lens), S, H)).astype(np.float64)
    xl = shift_left(xr, lens)
    layer = make_layer(W, heads, len(lens), S)
    got = layer.prefill(xl, lens, left_padded=True)                  # NaN pads: skipped, not masked
    want = bf.masked_layer(np.nan_to_num(xl, nan=0.5), lens, W, heads, left_padded=True)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(got[b, S - L:], want[b, S - L:], rtol=0, atol=1e-9)
        assert np.all(got[b, :S - L] == 0.0)
    # the padding side changes where rows live, nothing else: same numbers, same cache, same lengths
    k_left, v_left, n_left = layer.k_cache.copy(), layer.v_cache.copy(), layer.lens.copy()
    right = layer.prefill(xr, lens)
    for b, L in enumerate(lens):
        assert np.array_equal(got[b, S - L:], right[b, :L])
    assert np.array_equal(k_left, layer.k_cache, equal_nan=True) and np.array_equal(v_left, layer.v_cache, equal_nan=True)
    assert np.array_equal(n_left, layer.lens)


def test_left_padded_softmax_op_matches_additive_mask_bruteforce():
    lens, S = [9, 1, 5], 9
    s = wl.scores(21, 3, 2, S).astype(np.float64)
    got = orc.softmax_maskfree(s, lens, scale=0.7, left_padded=True)
    want = bf.masked_softmax(s, lens, scale=0.7, left_padded=True)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    for b, L in enumerate(lens):
        pad = S - L
        assert np.array_equal(got[b, :, :pad], s[b, :, :pad])            # rows of pad queries untouched
        assert np.all(got[b, :, pad:, :pad] == 0.0)                       # pad keys carry no weight
        assert np.all(np.triu(got[b, 0], 1)[pad:] == 0.0)                 # nor do later keys
        np.testing.assert_allclose(got[b, :, pad:].sum(-1), 1.0, atol=1e-12)
    # a window that starts at key 0 instead of padLen (pad keys visible) is a different function
    wrong = orc.softmax_maskfree(s, [S] * 3, scale=0.7)
    assert np.abs(wrong[1, :, S - 1] - want[1, :, S - 1]).max() > 1e-3


def test_left_padded_attention_op_equals_right_padded_shifted():
    lens, S, heads, d = [6, 3, 1], 6, 2, 4
    q, k, v = (wl.normal(31, t, (3, S, heads, d)).astype(np.float64) for t in (1, 2, 3))
    right = orc.attention_prefill(q, k, v, lens)
    left = orc.attention_prefill(shift_left(q, lens), shift_left(k, lens), shift_left(v, lens), lens, left_padded=True)
    for b, L in enumerate(lens):
        assert np.array_equal(left[b, S - L:], right[b, :L]) and np.all(left[b, :S - L] == 0.0)
