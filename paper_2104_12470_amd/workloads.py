"""Seeded synthetic inputs for the decoder-layer hot path.

This module produces *inputs only* (lengths, embeddings, weights); it holds none of the
method's arithmetic and imports neither the HIP binding nor the CPU oracle, so both sides
can be fed the same buffers.  The paper evaluates on fake inputs (Section 4, first
paragraph), so random tensors of the stated shapes are the paper's own workload.

Generator: a counter-based hash (splitmix64 finaliser) keyed by (seed, tensor id) gives
64 random bits per counter value; each counter makes one Box-Muller pair of normals.  Any
slice of any tensor can be regenerated without state, and the result does not depend on chunking.
"""
from __future__ import annotations

import os
from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = _mix64(np.array([(seed * 0x100000001B3 + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF], dtype=_U64))
        k = _mix64(k ^ (np.array([tensor_id & 0xFFFFFFFFFFFFFFFF], dtype=_U64) * _GOLD))
    return k[0]


def random_bits(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """64 random bits for counters start .. start+count-1 of stream (seed, tensor_id)."""
    key = _stream_key(seed, tensor_id)
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + count, dtype=_U64)
        return _mix64((ctr + _U64(1)) * _GOLD ^ key)


def uniform01(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in the open interval (0, 1), 53 random bits each."""
    bits = random_bits(seed, tensor_id, start, count)
    return ((bits >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_chunk(seed: int, tensor_id: int, lo: int, m: int, sigma: float, mean: float, out: np.ndarray) -> None:
    """Fill out[lo:lo+m] (m even or the tail).  Counter c yields elements 2c and 2c+1."""
    c0, c1 = lo // 2, (lo + m + 1) // 2
    bits = random_bits(seed, tensor_id, c0, c1 - c0)
    u1 = ((bits >> _U64(40)).astype(np.float32) + np.float32(0.5)) * np.float32(1.0 / 16777216.0)
    u2 = ((bits & _U64(0xFFFFFF)).astype(np.float32) + np.float32(0.5)) * np.float32(1.0 / 16777216.0)
    r = np.sqrt(np.float32(-2.0) * np.log(u1)) * np.float32(sigma)
    ang = np.float32(2.0 * np.pi) * u2
    z = np.empty(2 * (c1 - c0), dtype=np.float32)
    z[0::2] = r * np.cos(ang) + np.float32(mean)
    z[1::2] = r * np.sin(ang) + np.float32(mean)
    out[lo:lo + m] = z[lo - 2 * c0: lo - 2 * c0 + m].astype(out.dtype)


def normal(seed: int, tensor_id: int, shape, sigma: float = 1.0, mean: float = 0.0,
           dtype=np.float16, chunk: int = 1 << 22) -> np.ndarray:
    """Tensor of N(mean, sigma^2) samples (Box-Muller on 24-bit uniforms, float32 arithmetic),
    rounded to `dtype`.  Large tensors are filled by a thread pool; the values do not depend
    on the chunking."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    jobs = [(lo, min(chunk, n - lo)) for lo in range(0, n, chunk)]   # chunk is even
    if len(jobs) <= 1:
        for lo, m in jobs:
            _normal_chunk(seed, tensor_id, lo, m, sigma, mean, out)
    else:
        from concurrent.futures import ThreadPoolExecutor
        workers = min(len(jobs), max(1, len(os.sched_getaffinity(0))), 16)
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(lambda j: _normal_chunk(seed, tensor_id, j[0], j[1], sigma, mean, out), jobs))
    return out.reshape(shape)


def uniform_int(seed: int, tensor_id: int, count: int, lo: int, hi: int) -> np.ndarray:
    """`count` integers uniform on [lo, hi] inclusive (int32)."""
    u = uniform01(seed, tensor_id, 0, count)
    return np.minimum(lo + np.floor(u * (hi - lo + 1)), hi).astype(np.int32)


# --------------------------------------------------------------------------------------
# tensor ids inside one seed's stream family
# --------------------------------------------------------------------------------------
TID_LENS = 1
TID_PROMPT = 2
TID_DECODE = 3            # + step * 4096 + layer  (decode inputs are per step)
TID_LAYER_BASE = 1 << 20  # + layer * 64 + weight slot
TID_MODEL_HEAD = 1 << 19  # + slot (wte, wpe, lnf_g, lnf_b)
TID_PROMPT_IDS = 5
TID_DECODE_IDS = 6        # + step * 4096
_WEIGHT_SLOTS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: layer shape, batch shape and the seed it is drawn from."""
    name: str
    seed: int
    hidden: int
    heads: int
    ffn: int
    layers: int
    batch: int
    padded_len: int
    len_lo: int
    len_hi: int
    decode_steps: int
    max_seq: int
    sigma_w: float = 0.02
    tid_offset: int = 0     # separates workloads that share a seed
    ln_eps: float = 1e-5
    encoder: bool = False   # bidirectional use of the layer (no sequence mask, no decode)

    @property
    def d_head(self) -> int:
        return self.hidden // self.heads


# The five configurations the headline metric is defined on, plus tiny ones for unit tests.
WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("cfg1", 1001, 768, 12, 3072, 1, 4, 64, 16, 64, 0, 64),
    Workload("cfg2", 1002, 1024, 16, 4096, 24, 8, 512, 256, 512, 512, 1024),
    Workload("cfg3", 1003, 4096, 32, 16384, 1, 4, 1024, 512, 1024, 256, 1280),
    Workload("cfg4", 1004, 2048, 16, 8192, 1, 2, 4096, 2048, 4096, 128, 4224),
    Workload("cfg5a", 1005, 12288, 96, 49152, 1, 1, 2048, 2048, 2048, 64, 2112, sigma_w=0.006),
    Workload("cfg5b", 1005, 12288, 96, 49152, 1, 16, 2048, 1024, 2048, 64, 2112, sigma_w=0.006,
             tid_offset=1 << 16),
    # small shapes that still span several tiles and ragged tails
    Workload("tiny", 7, 64, 1, 256, 1, 3, 24, 1, 24, 4, 32),
    Workload("small64", 11, 256, 4, 1024, 2, 5, 200, 3, 200, 9, 224),
    Workload("small128", 13, 512, 4, 2048, 1, 3, 333, 40, 333, 7, 352),
    Workload("wide1280", 17, 1280, 10, 5120, 1, 3, 80, 20, 80, 5, 96),
    # encoder use (Section 4, Bert layer): hidden 1024, pad tokens about half of all tokens, no decode
    Workload("bert1024", 1006, 1024, 16, 4096, 24, 16, 256, 64, 192, 0, 256, encoder=True),
]}


def lengths(w: Workload) -> np.ndarray:
    """Valid prompt length per sequence, uniform on [len_lo, len_hi]."""
    return uniform_int(w.seed, w.tid_offset + TID_LENS, w.batch, w.len_lo, w.len_hi)


def prompt_embeddings(w: Workload, layer: int = 0) -> np.ndarray:
    """[batch, padded_len, hidden] fp16 ~ N(0,1); pad rows hold random values too."""
    return normal(w.seed, w.tid_offset + TID_PROMPT + layer * 8, (w.batch, w.padded_len, w.hidden))


def decode_embeddings(w: Workload, step: int, layer: int = 0) -> np.ndarray:
    """[batch, hidden] fp16 ~ N(0,1) fed at decode step `step` (independent of outputs)."""
    return normal(w.seed, w.tid_offset + TID_DECODE + step * 4096 + layer, (w.batch, w.hidden))


def layer_weights(w: Workload, layer: int = 0, random_affine: bool = False) -> Dict[str, np.ndarray]:
    """fp16 parameters of one decoder layer.

    Linear weights are row-major [out, in]; w_qkv stacks Q, K, V row blocks.  Weights and
    linear biases ~ N(0, sigma_w); LayerNorm gamma = 1, beta = 0 unless `random_affine`
    (then gamma ~ N(1, 0.1), beta ~ N(0, 0.1), used by parity sweeps).
    """
    H, F = w.hidden, w.ffn
    shapes = {"ln1_g": (H,), "ln1_b": (H,), "w_qkv": (3 * H, H), "b_qkv": (3 * H,),
              "w_o": (H, H), "b_o": (H,), "ln2_g": (H,), "ln2_b": (H,),
              "w_fc1": (F, H), "b_fc1": (F,), "w_fc2": (H, F), "b_fc2": (H,)}
    out = {}
    for slot, name in enumerate(_WEIGHT_SLOTS):
        tid = TID_LAYER_BASE + layer * 64 + slot  # weights are shared by workloads on one seed
        if name in ("ln1_g", "ln2_g"):
            out[name] = (normal(w.seed, tid, shapes[name], 0.1, 1.0) if random_affine
                         else np.ones(shapes[name], dtype=np.float16))
        elif name in ("ln1_b", "ln2_b"):
            out[name] = (normal(w.seed, tid, shapes[name], 0.1, 0.0) if random_affine
                         else np.zeros(shapes[name], dtype=np.float16))
        else:
            out[name] = normal(w.seed, tid, shapes[name], w.sigma_w)
    return out


def model_head(w: Workload, vocab: int, max_pos: int, random_affine: bool = False) -> Dict[str, np.ndarray]:
    """fp16 parameters around the stack: token embeddings wte [vocab, hidden] ~ N(0, 0.02) (also the output
    projection), position embeddings wpe [max_pos, hidden] ~ N(0, 0.01), final LayerNorm lnf_g / lnf_b."""
    H = w.hidden
    tid = w.tid_offset + TID_MODEL_HEAD
    return {"wte": normal(w.seed, tid, (vocab, H), 0.02), "wpe": normal(w.seed, tid + 1, (max_pos, H), 0.01),
            "lnf_g": normal(w.seed, tid + 2, (H,), 0.1, 1.0) if random_affine else np.ones(H, dtype=np.float16),
            "lnf_b": normal(w.seed, tid + 3, (H,), 0.1, 0.0) if random_affine else np.zeros(H, dtype=np.float16)}


def prompt_ids(w: Workload, vocab: int, pad_value: int = -1) -> np.ndarray:
    """[batch, padded_len] int32 token ids uniform on [0, vocab); entries past each sequence's length hold
    `pad_value` (out of range on purpose: nothing may read them)."""
    ids = uniform_int(w.seed, w.tid_offset + TID_PROMPT_IDS, w.batch * w.padded_len, 0, vocab - 1)
    ids = ids.reshape(w.batch, w.padded_len)
    for b, L in enumerate(lengths(w)):
        ids[b, int(L):] = pad_value
    return ids


def decode_ids(w: Workload, step: int, vocab: int) -> np.ndarray:
    """[batch] int32 token ids fed at decode step `step` when the generated tokens are not fed back."""
    return uniform_int(w.seed, w.tid_offset + TID_DECODE_IDS + step * 4096, w.batch, 0, vocab - 1)


def scores(seed: int, batch: int, heads: int, seq: int, sigma: float = 2.0) -> np.ndarray:
    """[batch, heads, seq, seq] fp16 raw attention scores for the stand-alone softmax op."""
    return normal(seed, 77, (batch, heads, seq, seq), sigma)


# ---- request / release sequences for the buffer manager (Section 3.2): inputs, no policy ----------------
ATTENTION_MODULE, FEED_FORWARD_MODULE = 0, 1


def unfused_layer_buffer_trace(batch: int, prompt: int, hidden: int, heads: int, ffn: int, elem_bytes: int = 2):
    """The buffers an unfused decoder layer asks for, in order, as ("req", name, bytes, module) and
    ("rel", name) events: a library GEMM for the stacked QKV projection, a kernel that adds the bias and splits
    heads into q, k, v, the materialised scores of Algorithm 1, the context and its head-merged copy, and the
    feed-forward intermediate.  Results that go to the activation caches (Section 3.1) are not buffers."""
    T = batch * prompt
    row = T * hidden * elem_bytes
    A, F = ATTENTION_MODULE, FEED_FORWARD_MODULE
    return [
        ("req", "qkv", 3 * row, A),
        ("req", "q", row, A), ("req", "k", row, A), ("req", "v", row, A),
        ("rel", "qkv"),
        ("req", "scores", batch * heads * prompt * prompt * elem_bytes, A),
        ("rel", "q"), ("rel", "k"),
        ("req", "ctx", row, A),
        ("rel", "v"), ("rel", "scores"),
        ("req", "ctx_merged", row, A),
        ("rel", "ctx"),
        ("rel", "ctx_merged"),
        ("req", "ffn1", T * ffn * elem_bytes, F),
        ("rel", "ffn1"),
    ]


def random_buffer_trace(seed: int, events: int, modules: int = 3, max_units: int = 12, unit: int = 256):
    """Seeded random requests (sizes of 1..max_units alignment units, minus a few bytes now and then) and
    releases of live buffers, as ("req", name, bytes, module) / ("rel", name) events."""
    r = uniform01(seed, 77, 0, 3 * events)
    out, live, n = [], [], 0
    for e in range(events):
        a, b, c = r[3 * e], r[3 * e + 1], r[3 * e + 2]
        if live and a < 0.45:
            out.append(("rel", live.pop(int(b * len(live)) % len(live))))
        else:
            size = (1 + int(b * max_units) % max_units) * unit - (int(c * 7) if c < 0.3 else 0)
            name = f"t{n}"
            n += 1
            out.append(("req", name, size, int(c * modules) % modules))
            live.append(name)
    return out
