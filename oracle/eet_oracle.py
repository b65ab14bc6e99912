"""CPU oracle for the mask-free decoder layer (EET, arXiv 2104.12470).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file: it is used by
`tests/`, by the smoke check and by the benchmark's CPU-baseline leg.  It shares no code
with the HIP library and does not import it.

What it computes.  Mask fusion (Section 2.1, Algorithm 1) replaces the additive attention
and padding masks by index comparisons; numerically the result is the ordinary pre-LN GPT-2
decoder layer evaluated on the valid tokens only.  The oracle is therefore that definition
written out, per sequence and per valid position, in float64:

    a  = LN(x_i)                         q,k,v = W_qkv a + b_qkv      (k,v stored in slot i)
    o  = per head: softmax_{j<=i}(q.k_j / sqrt(d)) applied to v_j     (keys 0..i inclusive)
    y  = x_i + W_o o + b_o
    z  = y + W_2 gelu(W_1 LN(y) + b_1) + b_2

Keys j > i, keys j >= L_b and query rows i >= L_b are never read (Section 2, first bullet:
padding tokens take no part; Section 2.1: a query sees only keys at or before its own
position).  The K/V cache follows Section 3.1: keys and values of every step are stored for
the next step, in storage sized once for the maximum batch and sequence length.

Readings of the paper taken here (the paper is silent or garbled on each):
  * sequences are right-padded: valid positions are [0, L_b); the paper's padLen is S - L_b;
  * the causal window includes the diagonal (key i is visible to query i);
  * pre-LN block, biases on all four linears, tanh-form GELU, eps = 1e-5, biased variance;
  * the 1/sqrt(d) scale is applied to the scores before the softmax;
  * output rows of pad positions are zero, and pad positions never touch the cache;
  * the stand-alone softmax (Algorithm 1 as an operator) writes zeros to the masked entries
    of valid rows and leaves pad rows unmodified.

Library primitives used as steps: numpy matmul for the dense projections, nothing else.
The attention is plain loops over (sequence, head, query row).

Pinned by tests/test_oracle_pins.py (brute force with explicit additive masks, causality and
padding-independence invariants, decode == prefill of the extended prompt, closed forms, a
float64 torch cross-check of the unpadded case, and the values the paper prints) and, for the
model around the stack, by tests/test_model_pins.py (hand-built tables, a float64 torch model of the
unpadded case, decode == prefill of the extended prompt, pad ids never read).
"""
from __future__ import annotations

import math
from typing import Dict, Iterable, List, Optional, Sequence

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# row-wise operators (Section 2.2 names them as the kernels that must span wide rows)
# --------------------------------------------------------------------------------------
def layernorm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """LayerNorm over the last axis: two-pass mean, biased variance."""
    x = np.asarray(x, F64)
    w = x.shape[-1]
    mu = x.sum(axis=-1, keepdims=True) / w
    dev = x - mu
    var = (dev * dev).sum(axis=-1, keepdims=True) / w
    return dev / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """GELU, tanh form (the one GPT-2 uses)."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x * x * x)))


def bias_gelu(x: np.ndarray, bias: np.ndarray) -> np.ndarray:
    """gelu(x + b) over rows of the feed-forward width."""
    return gelu_tanh(np.asarray(x, F64) + np.asarray(bias, F64))


def bias_residual(x: np.ndarray, bias: np.ndarray, residual: np.ndarray) -> np.ndarray:
    """x + b + residual (the residual connection of each sub-layer)."""
    return np.asarray(x, F64) + np.asarray(bias, F64) + np.asarray(residual, F64)


def linear(x: np.ndarray, w: np.ndarray, b: np.ndarray) -> np.ndarray:
    """y = x W^T + b with W stored [out, in]."""
    return np.asarray(x, F64) @ np.asarray(w, F64).T + np.asarray(b, F64)


def softmax_window(s: np.ndarray) -> np.ndarray:
    """Softmax of a 1-D score window (max-subtracted)."""
    m = s.max()
    e = np.exp(s - m)
    return e / e.sum()


# --------------------------------------------------------------------------------------
# Algorithm 1 as a stand-alone operator
# --------------------------------------------------------------------------------------
def softmax_maskfree(scores: np.ndarray, q_lens: Sequence[int], scale: float = 1.0,
                     left_padded: bool = False) -> np.ndarray:
    """Mask-free softmax over materialised scores [B, heads, S, S] (Algorithm 1).

    Right-padded (valid positions [0, L)): row i < L becomes softmax over keys 0..i and zero over
    keys i+1..S-1; rows i >= L (pad queries) are returned unchanged.
    left_padded: the layout Algorithm 1 is printed for.  With padLen = S - L, the row loop starts at the
    first non-pad position padLen and ends at the last token S-1, and the window of row i is
    padLen..i; entries of a valid row outside its window become zero, rows i < padLen are returned
    unchanged.
    """
    out = np.array(scores, dtype=F64, copy=True)
    B, nh, S, S2 = out.shape
    assert S == S2 and len(q_lens) == B
    for b in range(B):
        L = int(q_lens[b])
        first = S - L if left_padded else 0                 # first non-pad position
        for g in range(nh):
            for i in range(first, first + L):
                row = softmax_window(out[b, g, i, first: i + 1] * scale)
                out[b, g, i, :] = 0.0
                out[b, g, i, first: i + 1] = row
    return out


def padding_offsets(q_lens: Sequence[int], padded_len: int) -> Dict[str, np.ndarray]:
    """Integer by-products of the index set-up: the paper's padLen per sequence, and the
    prefix sums that place each sequence's valid rows in a packed token list."""
    q = np.asarray(q_lens, np.int64)
    cu = np.zeros(len(q) + 1, np.int64)
    cu[1:] = np.cumsum(q)
    return {"pad_len": (padded_len - q).astype(np.int32), "cu_seqlens": cu.astype(np.int32)}


# --------------------------------------------------------------------------------------
# attention over a K/V store, one query at a time
# --------------------------------------------------------------------------------------
def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, n_keys: int) -> np.ndarray:
    """Context vector of one query.

    q [heads, d]; K, V [heads, capacity, d]; keys 0 .. n_keys-1 are visible.
    """
    heads, d = q.shape
    o = np.empty((heads, d), F64)
    inv = 1.0 / math.sqrt(d)
    for g in range(heads):
        s = (K[g, :n_keys] @ q[g]) * inv
        p = softmax_window(s)
        o[g] = p @ V[g, :n_keys]
    return o


def attention_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_lens: Sequence[int],
                      causal: bool = True, left_padded: bool = False) -> np.ndarray:
    """Op-level padding-skipping attention.  q, k, v: [B, S, heads, d] (padded); returns the
    context [B, S, heads, d] with pad rows zero.  causal: query i sees keys 0..i (decoder);
    otherwise every valid query sees all L_b valid keys (the encoder layer of Section 4's
    Bert experiment: padding skip only, no sequence mask).  left_padded: the valid tokens of
    sequence b sit at positions S-L_b .. S-1 (the layout of Algorithm 1) instead of 0 .. L_b-1."""
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    B, S, nh, d = q.shape
    out = np.zeros_like(q)
    for b in range(B):
        L = int(q_lens[b])
        first = S - L if left_padded else 0
        Kb = np.ascontiguousarray(k[b, first: first + L].transpose(1, 0, 2))     # token t of the sequence at index t
        Vb = np.ascontiguousarray(v[b, first: first + L].transpose(1, 0, 2))
        for t in range(L):
            out[b, first + t] = attend(q[b, first + t], Kb, Vb, t + 1 if causal else L)
    return out


def attention_decode(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                     n_keys: Sequence[int]) -> np.ndarray:
    """Op-level incremental attention: q [B, heads, d]; caches [B, heads, capacity, d];
    sequence b sees its first n_keys[b] slots."""
    q = np.asarray(q, F64)
    out = np.empty_like(q)
    for b in range(q.shape[0]):
        out[b] = attend(q[b], np.asarray(k_cache[b], F64), np.asarray(v_cache[b], F64), int(n_keys[b]))
    return out


# --------------------------------------------------------------------------------------
# the decoder layer with its K/V cache
# --------------------------------------------------------------------------------------
class DecoderLayerOracle:
    """One pre-LN decoder layer plus its K/V cache (float64 throughout).

    `weights` maps ln1_g, ln1_b, w_qkv [3H,H], b_qkv, w_o [H,H], b_o, ln2_g, ln2_b,
    w_fc1 [F,H], b_fc1, w_fc2 [H,F], b_fc2 to arrays (any float dtype; widened exactly).
    """

    def __init__(self, weights: Dict[str, np.ndarray], heads: int, max_batch: int, max_seq: int,
                 eps: float = 1e-5):
        self.w = {k: np.asarray(v, F64) for k, v in weights.items()}
        self.H = self.w["w_o"].shape[0]
        self.F = self.w["w_fc1"].shape[0]
        self.heads = heads
        self.d = self.H // heads
        assert self.d * heads == self.H
        self.eps = eps
        self.max_batch, self.max_seq = max_batch, max_seq
        # cache slots that were never written stay NaN so that any stray read shows up
        self.k_cache = np.full((max_batch, heads, max_seq, self.d), np.nan, F64)
        self.v_cache = np.full((max_batch, heads, max_seq, self.d), np.nan, F64)
        self.lens = np.zeros(max_batch, np.int32)    # n_b
        self.batch = 0
        self.slot_log: List[np.ndarray] = []         # slot written per sequence, per decode step

    # ---- pieces -----------------------------------------------------------------------
    def _qkv(self, x: np.ndarray):
        a = layernorm(x, self.w["ln1_g"], self.w["ln1_b"], self.eps)
        qkv = linear(a, self.w["w_qkv"], self.w["b_qkv"])
        H = self.H
        shp = x.shape[:-1] + (self.heads, self.d)
        return qkv[..., :H].reshape(shp), qkv[..., H:2 * H].reshape(shp), qkv[..., 2 * H:].reshape(shp)

    def _after_attention(self, x: np.ndarray, ctx: np.ndarray) -> np.ndarray:
        y = x + linear(ctx, self.w["w_o"], self.w["b_o"])
        c = layernorm(y, self.w["ln2_g"], self.w["ln2_b"], self.eps)
        f = gelu_tanh(linear(c, self.w["w_fc1"], self.w["b_fc1"]))
        return y + linear(f, self.w["w_fc2"], self.w["b_fc2"])

    # ---- prefill ------------------------------------------------------------------------
    def prefill(self, x: np.ndarray, q_lens: Sequence[int],
                rows: Optional[Dict[int, Iterable[int]]] = None, causal: bool = True,
                left_padded: bool = False) -> np.ndarray:
        """Process whole prompts.  x [B, S, H]; q_lens[b] valid rows per sequence.

        left_padded: the valid rows of sequence b are x[b, S-L_b:] (the layout Algorithm 1 is printed
        for) instead of x[b, :L_b]; the result has the same layout.  Cache slots, `rows` and the
        lengths stay sequence-relative (slot t = token t of the sequence), so a decode step after
        either layout is the same computation.

        Returns [B, S, H] float64: valid rows hold the layer output, pad rows are zero.
        With `rows` = {b: positions}, only those query rows are evaluated (the cache is
        still filled for every valid token of the listed sequences); other valid rows of
        the result are NaN, and sequences not listed are left out of the cache.
        causal=False is the encoder use of the same layer: every valid row attends to all
        L_b valid tokens of its sequence (see encode()).
        """
        B, S, H = x.shape
        assert H == self.H and B <= self.max_batch and S <= self.max_seq and len(q_lens) == B
        out = np.zeros((B, S, H), F64)
        self.batch = B
        self.slot_log = []
        self.k_cache[...] = np.nan
        self.v_cache[...] = np.nan
        for b in range(B):
            L = int(q_lens[b])
            assert 1 <= L <= S
            self.lens[b] = L
            if rows is not None and b not in rows:
                out[b, (S - L if left_padded else 0):(S if left_padded else L)] = np.nan
                continue
            first = S - L if left_padded else 0
            xb = np.asarray(x[b, first: first + L], F64)    # pad rows are never read
            q, k, v = self._qkv(xb)                         # [L, heads, d]
            self.k_cache[b, :, :L] = k.transpose(1, 0, 2)   # slot i <- token i
            self.v_cache[b, :, :L] = v.transpose(1, 0, 2)
            want = range(L) if rows is None else sorted(set(int(i) for i in rows[b]))
            if rows is not None:
                out[b, first: first + L] = np.nan
            ctx = np.empty((len(want), H), F64)
            for r, i in enumerate(want):
                assert 0 <= i < L
                ctx[r] = attend(q[i], self.k_cache[b], self.v_cache[b], i + 1 if causal else L).reshape(H)
            idx = np.fromiter(want, dtype=np.int64, count=len(want))
            out[b, first + idx] = self._after_attention(xb[idx], ctx)
        return out

    def encode(self, x: np.ndarray, q_lens: Sequence[int],
               rows: Optional[Dict[int, Iterable[int]]] = None) -> np.ndarray:
        """The layer as a bidirectional encoder (Section 4, Bert layer experiment): the same
        block with the window predicate j <= i replaced by j < L_b.  Pad tokens are skipped,
        there is no sequence mask, and no decode step follows."""
        out = self.prefill(x, q_lens, rows, causal=False)
        self.batch = 0
        return out

    # ---- incremental decode -------------------------------------------------------------
    def decode_step(self, x: np.ndarray, seqs: Optional[Iterable[int]] = None) -> np.ndarray:
        """One new token per sequence: x [B, H] -> [B, H].  Token of sequence b goes to
        slot n_b, attends to slots 0..n_b, then n_b advances by one."""
        B, H = x.shape
        assert B == self.batch and H == self.H
        out = np.full((B, H), np.nan, F64)
        slots = self.lens[:B].copy()
        todo = range(B) if seqs is None else sorted(set(seqs))
        for b in todo:
            n = int(self.lens[b])
            assert n + 1 <= self.max_seq, "cache capacity exceeded"
            xb = np.asarray(x[b], F64)
            q, k, v = self._qkv(xb)
            self.k_cache[b, :, n] = k
            self.v_cache[b, :, n] = v
            ctx = attend(q, self.k_cache[b], self.v_cache[b], n + 1).reshape(H)
            out[b] = self._after_attention(xb, ctx)
        self.lens[:B] += 1
        self.slot_log.append(slots)
        return out


# --------------------------------------------------------------------------------------
# the model around the stack of layers (the model-level interface named in the Conclusion)
# --------------------------------------------------------------------------------------
# The paper names an embedding operator and a final output (Section 3.1, first bullet on activation
# caches) and GPT-2 as the model (Section 4) but prints none of their arithmetic.  Readings taken,
# all GPT-2's: the input of layer 0 is the token embedding plus a learned absolute position
# embedding; token t of a sequence has position t whatever the padding; after the last layer comes
# one more LayerNorm; the logits are that row times the transposed token-embedding matrix (any
# [vocab, hidden] matrix here), no bias; greedy decoding takes the first maximum.
def embedding(ids: Sequence[int], positions: Sequence[int], wte: np.ndarray, wpe: np.ndarray) -> np.ndarray:
    """Rows wte[id] + wpe[position], one per token.  Raises IndexError on an id or a position outside its table."""
    wte = np.asarray(wte, F64); wpe = np.asarray(wpe, F64)
    out = np.empty((len(ids), wte.shape[1]), F64)
    for r, (t, p) in enumerate(zip(ids, positions)):
        t = int(t); p = int(p)
        if not (0 <= t < wte.shape[0]) or not (0 <= p < wpe.shape[0]):
            raise IndexError(f"token {t} / position {p} outside the tables")
        out[r] = wte[t] + wpe[p]
    return out


def lm_head(x: np.ndarray, lnf_g: np.ndarray, lnf_b: np.ndarray, w_out: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """Logits of hidden rows x [rows, H]: LayerNorm, then the product with w_out^T (w_out [vocab, H])."""
    return layernorm(x, lnf_g, lnf_b, eps) @ np.asarray(w_out, F64).T


def greedy_token(logits: np.ndarray, vocab: Optional[int] = None) -> np.ndarray:
    """Index of the first maximum of each row over columns [0, vocab); a NaN never wins."""
    logits = np.asarray(logits, F64)
    vocab = logits.shape[-1] if vocab is None else vocab
    out = np.zeros(logits.shape[0], np.int32)
    for r in range(logits.shape[0]):
        best = -np.inf
        for j in range(vocab):
            if logits[r, j] > best:           # strict: the first of equal values stays; NaN compares false
                best = logits[r, j]
                out[r] = j
    return out


class DecoderModelOracle:
    """Embedding, a stack of decoder layers with their K/V caches, final LayerNorm and output projection.

    `layer_weights`: one dict per layer (see DecoderLayerOracle); `head`: wte [vocab, H], wpe [max_pos, H],
    lnf_g, lnf_b.  The output projection is wte itself (tied weights)."""

    def __init__(self, layer_weights: Sequence[Dict[str, np.ndarray]], head: Dict[str, np.ndarray], heads: int,
                 max_batch: int, max_seq: int, eps: float = 1e-5):
        self.layers = [DecoderLayerOracle(w, heads, max_batch, max_seq, eps) for w in layer_weights]
        self.head = {k: np.asarray(v, F64) for k, v in head.items()}
        self.eps = eps
        self.hidden_in = None        # input of layer 0 and output of the last layer of the latest call (for per-part checks)
        self.hidden_out = None

    def prefill(self, ids: np.ndarray, q_lens: Sequence[int], left_padded: bool = False) -> np.ndarray:
        """ids [B, S], q_lens[b] valid tokens: ids[b, :L_b] (right-padded) or, with left_padded, ids[b, S-L_b:] (the
        layout Algorithm 1 is printed for); pad entries are never read.  Token t of a sequence has position t in
        either layout.  Returns the logits [B, vocab] of the LAST valid token of every sequence (the ones the first
        generated token is drawn from)."""
        B, S = ids.shape
        H = self.head["wte"].shape[1]
        x = np.zeros((B, S, H), F64)
        first = [S - int(L) if left_padded else 0 for L in q_lens]
        for b in range(B):
            L = int(q_lens[b])
            x[b, first[b]: first[b] + L] = embedding(ids[b, first[b]: first[b] + L], range(L), self.head["wte"], self.head["wpe"])
        self.hidden_in = x
        for layer in self.layers:
            x = layer.prefill(x, q_lens, left_padded=left_padded)
        self.hidden_out = x
        last = np.stack([x[b, first[b] + int(q_lens[b]) - 1] for b in range(B)])
        return lm_head(last, self.head["lnf_g"], self.head["lnf_b"], self.head["wte"], self.eps)

    def decode_step(self, ids: Sequence[int]) -> np.ndarray:
        """One new token per sequence, at position n_b.  Returns its logits [B, vocab]."""
        pos = [int(n) for n in self.layers[0].lens[:len(ids)]]
        x = embedding(ids, pos, self.head["wte"], self.head["wpe"])
        self.hidden_in = x
        for layer in self.layers:
            x = layer.decode_step(x)
        self.hidden_out = x
        return lm_head(x, self.head["lnf_g"], self.head["lnf_b"], self.head["wte"], self.eps)


# --------------------------------------------------------------------------------------
# sizes and launch-shape rule printed in the paper
# --------------------------------------------------------------------------------------
def kv_cache_elements(max_batch: int, hidden: int, max_seq: int, layers: int = 1) -> int:
    """Section 3.1: the K/V caches hold 2 * b * h * s * l elements."""
    return 2 * max_batch * hidden * max_seq * layers


def activation_cache_elements(max_batch: int, hidden: int, max_prompt: int) -> int:
    """Section 3.1: the two activation caches hold 2 * b * h * p elements."""
    return 2 * max_batch * hidden * max_prompt


def buffer_elements(batch: int, prompt: int, hidden: int, heads: int) -> int:
    """Section 3.2: operator result buffers total b * p * (6h + n*p) elements."""
    return batch * prompt * (6 * hidden + heads * prompt)


def fold_shape(width: int, limit: int = 1024):
    """Thread-block folding (Section 2.2) as the text describes it: halve a virtual block
    of `width` threads until a piece fits the per-block limit.  Returns (pieces, threads
    per piece).  The printed closed form disagrees with the worked example in the same
    section; this follows the example and the stated 512-thread minimum."""
    pieces = 1
    while -(-width // pieces) > limit:
        pieces *= 2
    return pieces, -(-width // pieces)
