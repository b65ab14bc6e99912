"""Pins of the model-level oracle (embedding, final LayerNorm + output projection, greedy choice, the
model around the stack) against things other than itself.  CPU only."""
import numpy as np
import pytest

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl


def small_model(seed=31, H=32, heads=2, F=64, layers=2, vocab=19, max_pos=12, B=3, S=9, lo=2, hi=9, affine=True):
    w = wl.Workload("m", seed, H, heads, F, layers, B, S, lo, hi, 3, max_pos, sigma_w=0.2)
    LW = [{k: v.astype(np.float64) for k, v in wl.layer_weights(w, l, random_affine=affine).items()} for l in range(layers)]
    head = {k: v.astype(np.float64) for k, v in wl.model_head(w, vocab, max_pos, random_affine=affine).items()}
    head["wte"] = head["wte"] * 20.0      # embeddings of order 0.4 so that no term of the sum is negligible
    head["wpe"] = head["wpe"] * 30.0
    return w, LW, head


# ------------------------------------------------------------------ embedding: hand-built tables
def test_embedding_reads_the_row_of_the_token_and_the_row_of_the_position():
    V, P, H = 7, 5, 12
    wte = np.zeros((V, H)); wpe = np.zeros((P, H))
    for v in range(V):
        wte[v, v] = 1.0 + v                # token v marks column v
    for p in range(P):
        wpe[p, V + p] = 100.0 + p          # position p marks column V + p
    ids, pos = [3, 0, 6, 3], [0, 4, 2, 1]
    x = orc.embedding(ids, pos, wte, wpe)
    for r in range(4):
        want = np.zeros(H)
        want[ids[r]] = 1.0 + ids[r]
        want[V + pos[r]] = 100.0 + pos[r]
        assert np.array_equal(x[r], want)
    with pytest.raises(IndexError):
        orc.embedding([7], [0], wte, wpe)
    with pytest.raises(IndexError):
        orc.embedding([-1], [0], wte, wpe)
    with pytest.raises(IndexError):
        orc.embedding([0], [5], wte, wpe)


# ------------------------------------------------------------------ greedy choice: brute force and ties
def test_greedy_token_is_the_first_maximum_of_the_valid_columns():
    lg = np.array([[0.5, 2.0, 2.0, -1.0, 9.0],       # the 9 sits in a padding column
                   [-3.0, -3.0, -7.0, -3.0, 0.0],
                   [np.nan, 1.0, np.nan, 4.0, 4.0],
                   [-np.inf, -np.inf, -5.0, -np.inf, 1.0]])
    assert orc.greedy_token(lg, vocab=4).tolist() == [1, 0, 3, 2]
    assert orc.greedy_token(lg).tolist() == [4, 4, 3, 4]
    r = wl.normal(3, 9, (50, 33)).astype(np.float64)
    assert np.array_equal(orc.greedy_token(r), np.argmax(r, axis=1))


# ------------------------------------------------------------------ output projection: library special case
def test_lm_head_matches_torch_float64():
    torch = pytest.importorskip("torch")
    Fn = torch.nn.functional
    x = wl.normal(8, 1, (5, 48)).astype(np.float64)
    g = wl.normal(8, 2, (48,), 0.1, 1.0).astype(np.float64); b = wl.normal(8, 3, (48,), 0.1).astype(np.float64)
    w = wl.normal(8, 4, (23, 48), 0.3).astype(np.float64)
    want = Fn.linear(Fn.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), 1e-5), torch.from_numpy(w))
    np.testing.assert_allclose(orc.lm_head(x, g, b, w), want.numpy(), rtol=0, atol=1e-12)


def test_lm_head_closed_form_orthogonal_rows():
    # w rows = signed unit vectors, gamma = 1, beta = 0: the logit of row v is the normalised x[v] itself
    H = 16
    x = wl.normal(9, 1, (4, H)).astype(np.float64)
    lg = orc.lm_head(x, np.ones(H), np.zeros(H), np.eye(H))
    n = (x - x.mean(1, keepdims=True)) / np.sqrt(x.var(1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(lg, n, rtol=0, atol=1e-12)
    assert np.array_equal(orc.greedy_token(lg), np.argmax(x, axis=1))


# ------------------------------------------------------------------ the whole model: library special case
def test_unpadded_model_matches_torch_float64():
    torch = pytest.importorskip("torch")
    Fn = torch.nn.functional
    w, LW, head = small_model(B=2, S=9, lo=9, hi=9)
    H, heads, B, S = w.hidden, w.heads, w.batch, w.padded_len
    d = H // heads
    ids = wl.prompt_ids(w, 19)
    m = orc.DecoderModelOracle(LW, head, heads, B, w.max_seq)
    got = m.prefill(ids, [S] * B)
    T = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    x = Fn.embedding(torch.from_numpy(ids.astype(np.int64)), T(head["wte"])) + T(head["wpe"])[:S].unsqueeze(0)
    np.testing.assert_allclose(m.hidden_in, x.numpy(), rtol=0, atol=0)
    for W in LW:
        a = Fn.layer_norm(x, (H,), T(W["ln1_g"]), T(W["ln1_b"]), 1e-5)
        qkv = Fn.linear(a, T(W["w_qkv"]), T(W["b_qkv"])).view(B, S, 3, heads, d).permute(2, 0, 3, 1, 4)
        ctx = Fn.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2], is_causal=True)
        y = x + Fn.linear(ctx.transpose(1, 2).reshape(B, S, H), T(W["w_o"]), T(W["b_o"]))
        c = Fn.layer_norm(y, (H,), T(W["ln2_g"]), T(W["ln2_b"]), 1e-5)
        x = y + Fn.linear(Fn.gelu(Fn.linear(c, T(W["w_fc1"]), T(W["b_fc1"])), approximate="tanh"), T(W["w_fc2"]), T(W["b_fc2"]))
    logits = Fn.linear(Fn.layer_norm(x[:, -1], (H,), T(head["lnf_g"]), T(head["lnf_b"]), 1e-5), T(head["wte"]))
    np.testing.assert_allclose(got, logits.numpy(), rtol=0, atol=1e-9)


# ------------------------------------------------------------------ invariants of the ragged, cached case
def test_model_decode_equals_prefill_of_the_extended_prompt_and_positions_follow_the_cache_length():
    w, LW, head = small_model()
    lens = [int(v) for v in wl.lengths(w)]
    B, S = w.batch, w.padded_len
    ids = wl.prompt_ids(w, 19)
    m = orc.DecoderModelOracle(LW, head, w.heads, B, w.max_seq)
    m.prefill(ids, lens)
    steps = [wl.decode_ids(w, k, 19) for k in range(3)]
    for k, nxt in enumerate(steps):
        got = m.decode_step(nxt)
        for b in range(B):      # the same tokens as one longer prompt, sequence by sequence (no padding at all)
            full = np.concatenate([ids[b, :lens[b]], [s[b] for s in steps[:k + 1]]]).astype(np.int32)[None, :]
            ref = orc.DecoderModelOracle(LW, head, w.heads, 1, w.max_seq).prefill(full, [full.shape[1]])
            np.testing.assert_allclose(got[b], ref[0], rtol=0, atol=1e-9)
    assert m.layers[0].lens[:B].tolist() == [L + 3 for L in lens]


def test_pad_ids_are_never_read_and_each_sequence_is_independent():
    w, LW, head = small_model()
    lens = [int(v) for v in wl.lengths(w)]
    ids = wl.prompt_ids(w, 19, pad_value=-1)          # any read of a pad entry raises IndexError in the oracle
    assert any(L < w.padded_len for L in lens)
    m = orc.DecoderModelOracle(LW, head, w.heads, w.batch, w.max_seq)
    a = m.prefill(ids, lens)
    ids2 = wl.prompt_ids(w, 19, pad_value=10 ** 6)
    ids2[0, :lens[0]] = (ids2[0, :lens[0]] + 1) % 19   # another prompt for sequence 0
    b = orc.DecoderModelOracle(LW, head, w.heads, w.batch, w.max_seq).prefill(ids2, lens)
    assert np.array_equal(a[1:], b[1:])
    assert not np.allclose(a[0], b[0])


def test_position_embedding_matters_and_is_sequence_relative():
    # a one-token prompt sits at position 0: its hidden input is wte[id] + wpe[0], whatever the row is padded to
    w, LW, head = small_model(B=1, S=6, lo=1, hi=1)
    m = orc.DecoderModelOracle(LW, head, w.heads, 1, w.max_seq)
    ids = np.full((1, 6), -1, np.int32); ids[0, 0] = 4
    m.prefill(ids, [1])
    assert np.array_equal(m.hidden_in[0, 0], head["wte"][4] + head["wpe"][0])
    m.decode_step([7])
    assert np.array_equal(m.hidden_in[0], head["wte"][7] + head["wpe"][1])


def test_left_padded_model_equals_the_right_padded_one():
    # same tokens, pads in front: embedding rows move to the end of each row block with the same values (positions are
    # sequence-relative), logits, cache and lengths are bitwise those of the right-padded call
    w, LW, head = small_model()
    lens = [int(v) for v in wl.lengths(w)]
    B, S = w.batch, w.padded_len
    ids = wl.prompt_ids(w, 19, pad_value=-1)
    left = np.full_like(ids, -1)
    for b, L in enumerate(lens):
        left[b, S - L:] = ids[b, :L]
    a = orc.DecoderModelOracle(LW, head, w.heads, B, w.max_seq)
    c = orc.DecoderModelOracle(LW, head, w.heads, B, w.max_seq)
    la, lc = a.prefill(ids, lens), c.prefill(left, lens, left_padded=True)
    assert np.array_equal(la, lc)
    for b, L in enumerate(lens):
        assert np.array_equal(a.hidden_in[b, :L], c.hidden_in[b, S - L:])
        assert np.all(c.hidden_in[b, :S - L] == 0) and np.all(c.hidden_out[b, :S - L] == 0)
        assert np.array_equal(a.hidden_out[b, :L], c.hidden_out[b, S - L:])
        assert np.array_equal(c.hidden_in[b, S - L], head["wte"][ids[b, 0]] + head["wpe"][0])     # first token: position 0
    nxt = wl.decode_ids(w, 0, 19)
    assert np.array_equal(a.decode_step(nxt), c.decode_step(nxt))
    assert a.layers[0].lens.tolist() == c.layers[0].lens.tolist()


# ------------------------------------------------------------------ planted mistakes must fail a pin
def test_planted_mistakes_in_the_model_fail_the_pins(monkeypatch):
    w, LW, head = small_model(B=1, S=6, lo=3, hi=3)
    ids = wl.prompt_ids(w, 19)
    good = orc.DecoderModelOracle(LW, head, w.heads, 1, w.max_seq).prefill(ids, [3])
    # (1) positions off by one, (2) no final LayerNorm: each changes the logits by far more than the pins' tolerances
    def emb_off_by_one(i, p, wte, wpe):
        return np.asarray(wte)[list(i)] + np.asarray(wpe)[[q + 1 for q in p]]
    monkeypatch.setattr(orc, "embedding", emb_off_by_one)
    bad = orc.DecoderModelOracle(LW, head, w.heads, 1, w.max_seq).prefill(ids, [3])
    assert np.abs(bad - good).max() > 1e-3
    monkeypatch.undo()
    monkeypatch.setattr(orc, "lm_head", lambda x, g, b, wo, eps=1e-5: np.asarray(x) @ np.asarray(wo).T)
    bad = orc.DecoderModelOracle(LW, head, w.heads, 1, w.max_seq).prefill(ids, [3])
    assert np.abs(bad - good).max() > 1e-3
