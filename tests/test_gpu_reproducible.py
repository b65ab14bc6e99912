"""Run-to-run reproducibility at full size, once per suite.

The path uses no floating-point atomics and fixes every reduction order, so two runs of the same calls on two fresh
handles must agree bit for bit -- in the result AND in everything they leave behind.  Each case runs the same calls on
two handles whose workspaces start out zeroed and compares, byte for byte, the outputs of every call, every layer's
K/V region and the whole workspace, whose pieces are the intermediate results of the last layer that ran (attention
context, output-projection result, normalised rows, feed-forward activations) and the stack's two activation buffers.
A difference is reported with the first differing piece, so it names the kernel that produced it.

Cases reach the paths the small workloads do not: 256x256 tiles, 128x64 and 64x64 tiles with two K groups, the
prefetch workgroups of small-layer decode, decode steps replayed from the stack's graph, the 256-row attention."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2104_12470_amd import workloads as wl
from tests.gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def first_difference(a: torch.Tensor, b: torch.Tensor):
    """None when the two byte buffers are equal, else (count, first byte offset)."""
    a8, b8 = a.reshape(-1).view(torch.uint8), b.reshape(-1).view(torch.uint8)
    if torch.equal(a8, b8):
        return None
    diff = (a8 != b8).nonzero()
    return int(diff.numel()), int(diff[0])


def workspace_piece(w, max_batch, offset):
    """Name of the workspace piece a byte offset falls in (the carve-up of csrc/eet_api.hip: lengths, prefix sums, row
    map, then the [T, H] buffers A, B, Y, the [T, F] buffer, the decode partials, and for a stack the two activation
    buffers)."""
    al = lambda v: (v + 255) // 256 * 256
    T, H, F = max_batch * w.padded_len, w.hidden, w.ffn
    pieces = [("cache lengths", al(4 * 128)), ("prefix sums", al(4 * 129)), ("row map", al(4 * T)),
              ("buffer A: LayerNorm-1 rows, then the attention context", al(2 * T * H)),
              ("buffer B: Q rows, then LayerNorm-2 rows", al(2 * T * H)),
              ("buffer Y: output projection + residual", al(2 * T * H)),
              ("buffer F: first feed-forward projection + GELU", al(2 * T * (F + 64)))]   # room for rows 128 bytes further apart
    lo = 0
    for name, size in pieces:
        if offset < lo + size:
            return f"{name} (+{offset - lo} bytes)"
        lo += size
    return f"decode partials / stack activation buffers (+{offset - lo} bytes past the layer buffers)"


def run_stack(eet, w, LW, steps):
    cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
    st = eet.DecoderStack(cfg, LW, use_graph=True)
    st.workspace.zero_()
    torch.cuda.synchronize()
    lens = [int(v) for v in wl.lengths(w)]
    stream = torch.cuda.Stream()
    outs = []
    with torch.cuda.stream(stream):
        outs.append(st.prefill(dev(wl.prompt_embeddings(w)), lens, stream=stream).clone())
        tok = torch.empty((w.batch, w.hidden), dtype=torch.float16, device="cuda:0")
        out = torch.empty_like(tok)
        for k in range(steps):                      # fixed buffers: steps 1.. replay the graph recorded by step 0
            tok.copy_(dev(wl.decode_embeddings(w, k)))
            st.decode_step(tok, out, stream=stream)
            outs.append(out.clone())
    stream.synchronize()
    torch.cuda.synchronize()
    return st, outs


@pytest.mark.parametrize("name,batch,layers", [("cfg2", 8, 24),      # 256x256 and 128x64 tiles, prefetch workgroups, graph
                                               ("cfg2", 2, 4)])      # 128x64 and 64x64 tiles with two K groups
def test_stack_runs_are_bitwise_reproducible_at_full_size(eet, name, batch, layers):
    w = replace(wl.WORKLOADS[name], batch=batch, layers=layers)
    LW = [{k: torch.from_numpy(v) for k, v in wl.layer_weights(w, l).items()} for l in range(layers)]
    print(f"reproducibility: {name} batch {batch}, {layers} layers, prefill + 3 graph-replayed decode steps, two handles", flush=True)
    a, outs_a = run_stack(eet, w, LW, 3)
    b, outs_b = run_stack(eet, w, LW, 3)
    what = f"{name} batch {batch} x {layers} layers"
    for i, (x, y) in enumerate(zip(outs_a, outs_b)):
        d = first_difference(x, y)
        assert d is None, f"{what}: output of {'the prefill' if i == 0 else f'decode step {i - 1}'} differs in {d[0]} bytes, first at {d[1]}"
    per_layer = a.kv_cache.numel() // layers
    for l in range(layers):
        d = first_difference(a.kv_cache[l * per_layer:(l + 1) * per_layer], b.kv_cache[l * per_layer:(l + 1) * per_layer])
        assert d is None, (f"{what}: K/V region of layer {l} differs in {d[0]} bytes, first at byte {d[1]} "
                           f"({'K' if d[1] < per_layer else 'V'} half): the input of layer {l} or its QKV projection")
    d = first_difference(a.workspace, b.workspace)
    assert d is None, f"{what}: workspace differs in {d[0]} bytes, first in {workspace_piece(w, w.batch, d[1])}"
    assert a.cache_lens(batch) == b.cache_lens(batch)
    a.close()
    b.close()


@pytest.mark.parametrize("name", ["cfg3"])               # 256x256 tiles, 256-row attention, weight-streaming decode
def test_layer_runs_are_bitwise_reproducible_at_full_size(eet, name):
    w = wl.WORKLOADS[name]
    W = {k: torch.from_numpy(v) for k, v in wl.layer_weights(w).items()}
    lens = [int(v) for v in wl.lengths(w)]
    x = dev(wl.prompt_embeddings(w))
    xs = [dev(wl.decode_embeddings(w, k)) for k in range(3)]
    print(f"reproducibility: {name} layer, prefill + 3 decode steps, two handles", flush=True)
    runs = []
    for _ in range(2):
        cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
        layer = eet.DecoderLayer(cfg, W)
        layer.workspace.zero_()
        torch.cuda.synchronize()
        outs = [layer.prefill(x, lens).clone()]
        torch.cuda.synchronize()
        after_prefill = layer.workspace.clone()
        for k in range(3):
            outs.append(layer.decode_step(xs[k]).clone())
        torch.cuda.synchronize()
        runs.append((layer, outs, after_prefill))
    (la, oa, wa), (lb, ob, wb) = runs
    d = first_difference(wa, wb)
    assert d is None, f"{name}: workspace after the prefill differs in {d[0]} bytes, first in {workspace_piece(w, w.batch, d[1])}"
    for i, (p, q) in enumerate(zip(oa, ob)):
        d = first_difference(p, q)
        assert d is None, f"{name}: output of {'the prefill' if i == 0 else f'decode step {i - 1}'} differs in {d[0]} bytes, first at {d[1]}"
    d = first_difference(la.kv_cache, lb.kv_cache)
    assert d is None, f"{name}: K/V cache differs in {d[0]} bytes, first at {d[1]}"
    d = first_difference(la.workspace, lb.workspace)
    assert d is None, f"{name}: workspace after the decode steps differs in {d[0]} bytes, first in {workspace_piece(w, w.batch, d[1])}"
    la.close()
    lb.close()
