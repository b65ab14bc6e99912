"""Brute-force masked decoder layer, used only to pin the oracle on tiny inputs.

Deliberately the *other* formulation: every sequence is processed at the padded length,
dense S x S scores are formed for all rows (pad rows included), and explicit additive masks
(-inf above the diagonal, -inf on pad key columns) are added before a dense softmax --
exactly what mask fusion (Section 2.1 of the paper) says it replaces.  Scalar Python loops
and math.* calls only, no shared helpers with the oracle.
"""
import math

import numpy as np


def _ln(row, g, b, eps):
    n = len(row)
    mu = sum(row) / n
    var = sum((t - mu) ** 2 for t in row) / n
    return [(t - mu) / math.sqrt(var + eps) * g[c] + b[c] for c, t in enumerate(row)]


def _matvec(w, bias, vec):
    return [sum(w[o][c] * vec[c] for c in range(len(vec))) + bias[o] for o in range(len(w))]


def _gelu(t):
    return 0.5 * t * (1.0 + math.tanh(0.7978845608028654 * (t + 0.044715 * t ** 3)))


def masked_layer(x, q_lens, W, heads, eps=1e-5, causal_mask=True, left_padded=False):
    """x [B,S,H] -> [B,S,H]; rows of pad positions are returned as zeros.  causal_mask=False
    drops the -inf triangle and keeps only the padding mask (the bidirectional encoder).
    left_padded: the pad positions are the first S-L of a sequence instead of the last."""
    x = np.asarray(x, np.float64)
    B, S, H = x.shape
    d = H // heads
    Wl = {k: np.asarray(v, np.float64).tolist() for k, v in W.items()}
    out = np.zeros((B, S, H))
    NEG = float("-inf")
    for b in range(B):
        L = int(q_lens[b])
        # finite stand-in for pad rows: an additive mask cannot cancel NaN/Inf, so a masked
        # implementation needs finite pad content; its value must not matter.
        valid = [(i >= S - L) if left_padded else (i < L) for i in range(S)]
        rows = [x[b, i].tolist() if valid[i] else [0.25] * H for i in range(S)]
        qkv = [_matvec(Wl["w_qkv"], Wl["b_qkv"], _ln(r, Wl["ln1_g"], Wl["ln1_b"], eps)) for r in rows]
        causal = [[0.0 if (j <= i or not causal_mask) else NEG for j in range(S)] for i in range(S)]
        padmask = [0.0 if valid[j] else NEG for j in range(S)]
        ctx = [[0.0] * H for _ in range(S)]
        for g in range(heads):
            lo = g * d
            for i in range(S):
                sc = []
                for j in range(S):
                    dot = sum(qkv[i][lo + c] * qkv[j][H + lo + c] for c in range(d))
                    sc.append(dot / math.sqrt(d) + causal[i][j] + padmask[j])
                m = max(sc)
                e = [math.exp(t - m) for t in sc]
                z = sum(e)
                for c in range(d):
                    ctx[i][lo + c] = sum(e[j] / z * qkv[j][2 * H + lo + c] for j in range(S))
        for i in range(S):
            if not valid[i]:
                continue
            att = _matvec(Wl["w_o"], Wl["b_o"], ctx[i])
            y = [rows[i][c] + att[c] for c in range(H)]
            f = [_gelu(t) for t in _matvec(Wl["w_fc1"], Wl["b_fc1"], _ln(y, Wl["ln2_g"], Wl["ln2_b"], eps))]
            z2 = _matvec(Wl["w_fc2"], Wl["b_fc2"], f)
            out[b, i] = [y[c] + z2[c] for c in range(H)]
    return out


def masked_softmax(scores, q_lens, scale=1.0, left_padded=False):
    """Dense additive-mask softmax of [B,nh,S,S]; returns probabilities for valid rows and the
    input unchanged for pad rows."""
    s = np.asarray(scores, np.float64)
    B, nh, S, _ = s.shape
    out = s.copy()
    for b in range(B):
        L = int(q_lens[b])
        mask = np.zeros((S, S))
        mask[np.triu_indices(S, 1)] = -np.inf
        lo, hi = (S - L, S) if left_padded else (0, L)
        mask[:, :lo] = -np.inf
        mask[:, hi:] = -np.inf
        for g in range(nh):
            t = s[b, g] * scale + mask
            with np.errstate(invalid="ignore"):              # rows of pad queries can be all -inf: they are not used
                t = t - t.max(axis=1, keepdims=True)
                e = np.exp(t)
                p = e / e.sum(axis=1, keepdims=True)
            out[b, g, lo:hi] = p[lo:hi]
    return out
