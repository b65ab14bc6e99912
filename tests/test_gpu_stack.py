"""The stack entry points (all layers per call, decode steps replayed from a HIP graph) against the
per-layer entry points and against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl
from tests.gpu_util import dev, gate, host

pytestmark = pytest.mark.gpu

SENTINEL = 777.0


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def build(eet, w, n_layers, use_graph):
    cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
    Ws = [wl.layer_weights(w, li, random_affine=True) for li in range(n_layers)]
    tw = [{k: torch.from_numpy(v) for k, v in W.items()} for W in Ws]
    return cfg, Ws, eet.DecoderStack(cfg, tw, cache_fill=SENTINEL, use_graph=use_graph)


@pytest.mark.parametrize("name,n_layers", [("small64", 2), ("small128", 3)])
def test_stack_equals_layer_chain_and_oracle(eet, name, n_layers):
    w = wl.WORKLOADS[name]
    cfg, Ws, stack = build(eet, w, n_layers, use_graph=False)
    lens, x = wl.lengths(w), wl.prompt_embeddings(w)
    B = w.batch
    layers = [eet.DecoderLayer(cfg, {k: torch.from_numpy(v) for k, v in W.items()}) for W in Ws]
    oracles = [orc.DecoderLayerOracle(W, w.heads, B, w.max_seq, w.ln_eps) for W in Ws]

    got = stack.prefill(dev(x), lens)
    h, ho = dev(x), x.astype(np.float64)
    for layer, o in zip(layers, oracles):
        h = layer.prefill(h, lens)
        ho = o.prefill(ho, lens)
    torch.cuda.synchronize()
    assert np.array_equal(host(got).view(np.uint16), host(h).view(np.uint16))          # same kernels, same bits
    for b, L in enumerate(lens):
        gate(host(got)[b, :L], ho[b, :L], f"{name} stack prefill b={b}")
        assert np.all(host(got)[b, L:] == 0)
    for k in range(4):
        xs = wl.decode_embeddings(w, k)
        got = stack.decode_step(dev(xs))
        h, ho = dev(xs), xs.astype(np.float64)
        for layer, o in zip(layers, oracles):
            h = layer.decode_step(h)
            ho = o.decode_step(ho)
        torch.cuda.synchronize()
        assert np.array_equal(host(got).view(np.uint16), host(h).view(np.uint16))
        gate(host(got), ho, f"{name} stack decode {k}")
        assert stack.cache_lens(B) == [int(v) + k + 1 for v in lens] == oracles[0].lens[:B].tolist()
    for li, o in enumerate(oracles):                                                     # per-layer caches, exact extents
        kc, vc = stack.cache_views(li)
        for b in range(B):
            n = int(lens[b]) + 4
            gate(host(kc[b, :, :n]), o.k_cache[b, :, :n], f"layer {li} K", 1.5e-2, 1.5e-3)
            assert bool((kc[b, :, n:] == SENTINEL).all()) and bool((vc[b, :, n:] == SENTINEL).all())
    stack.close()
    for layer in layers:
        layer.close()


def test_graph_replay_matches_direct_launches(eet):
    """Decode steps replayed from the recorded graph, with unrelated eager work and synchronisations
    between the replays, give the same bits as direct launches, step after step; a new prefill with
    another batch size re-records the graph."""
    w = wl.WORKLOADS["small64"]
    cfg, Ws, direct = build(eet, w, 2, use_graph=False)
    _, _, graphed = build(eet, w, 2, use_graph=True)
    side = torch.cuda.Stream()
    x = dev(wl.prompt_embeddings(w))
    tok = torch.empty((w.batch, w.hidden), dtype=torch.float16, device="cuda:0")      # fixed input buffer
    out_g = torch.empty_like(tok)
    for lens in ([int(v) for v in wl.lengths(w)], [7, 150, 64]):
        B = len(lens)
        with torch.cuda.stream(side):
            direct.prefill(x[:B], lens)
            graphed.prefill(x[:B], lens)
            for k in range(6):
                xs = dev(wl.decode_embeddings(w, k)[:B])
                tok[:B].copy_(xs)
                want = direct.decode_step(xs)
                graphed.decode_step(tok[:B], out_g[:B])
                side.synchronize()
                assert np.array_equal(host(out_g[:B]).view(np.uint16), host(want).view(np.uint16)), (B, k)
                assert graphed.cache_lens(B) == direct.cache_lens(B) == [v + k + 1 for v in lens]
                junk = torch.randn(257, 129, device="cuda:0").softmax(-1).sum()                 # eager work in between
                torch.cuda.synchronize()
                assert float(junk) > 0
    direct.close()
    graphed.close()


def test_stack_capacity(eet):
    w = wl.WORKLOADS["tiny"]
    cfg, Ws, stack = build(eet, w, 2, use_graph=True)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        stack.prefill(dev(wl.prompt_embeddings(w)), [24, 3, 1])
        xs = dev(wl.decode_embeddings(w, 0))
        o = torch.empty_like(xs)
        for _ in range(8):
            stack.decode_step(xs, o)
        side.synchronize()
        assert stack.cache_lens(3) == [32, 11, 9]
        with pytest.raises(eet.EETError) as e:
            stack.decode_step(xs, o)
        assert e.value.code == eet.EET_ERR_CAPACITY
        assert stack.cache_lens(3) == [32, 11, 9]
    stack.close()


def shift_to_the_end(x, lens):
    """Right-padded [B, S, ...] -> left-padded: the valid rows of sequence b moved to the end of its block, NaN in front."""
    out = np.full_like(x, np.nan)
    S = x.shape[1]
    for b, L in enumerate(lens):
        out[b, S - int(L):] = x[b, :int(L)]
    return out


@pytest.mark.parametrize("name,n_layers", [("small64", 2), ("small128", 3)])
def test_left_padded_stack_prefill(eet, name, n_layers):
    """Pads in front (the layout Algorithm 1 is printed for), through every layer: the valid rows are bit for bit those
    of the right-padded call, shifted; the caches and lengths are identical, and so is the decode step that follows;
    the pad rows (NaN on input) are zeros on output; against the oracle's left-padded stack within the layer tolerance."""
    w = wl.WORKLOADS[name]
    cfg, Ws, right = build(eet, w, n_layers, use_graph=False)
    _, _, left = build(eet, w, n_layers, use_graph=True)
    lens, x = wl.lengths(w), wl.prompt_embeddings(w)
    B, S = w.batch, w.padded_len
    xl = shift_to_the_end(x, lens)
    stream = torch.cuda.Stream()
    got_r = right.prefill(dev(x), lens)
    with torch.cuda.stream(stream):
        got_l = left.prefill_left_padded(dev(xl), lens, stream=stream)
    torch.cuda.synchronize()
    ho = xl.astype(np.float64)
    oracles = [orc.DecoderLayerOracle(W, w.heads, B, w.max_seq, w.ln_eps) for W in Ws]
    for o in oracles:
        ho = o.prefill(ho, lens, left_padded=True)
    gr, gl = host(got_r), host(got_l)
    for b, L in enumerate(lens):
        L = int(L)
        assert np.array_equal(gl[b, S - L:].view(np.uint16), gr[b, :L].view(np.uint16))
        assert np.all(gl[b, :S - L] == 0)
        gate(gl[b, S - L:], ho[b, S - L:], f"{name} left-padded stack b={b}")
    assert left.cache_lens(B) == right.cache_lens(B) == [int(v) for v in lens]
    assert torch.equal(left.kv_cache, right.kv_cache)
    xs = wl.decode_embeddings(w, 0)
    d_r = right.decode_step(dev(xs))
    with torch.cuda.stream(stream):
        d_l = left.decode_step(dev(xs), stream=stream)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_l).view(np.uint16), host(d_r).view(np.uint16))
    assert torch.equal(left.kv_cache, right.kv_cache)
    left.close()
    right.close()


@pytest.mark.parametrize("name,n_layers", [("small64", 2), ("small128", 3)])
def test_stack_encode_equals_layer_chain_and_oracle(eet, name, n_layers):
    """All layers as a bidirectional encoder in one call: bit for bit the chain of eet_layer_encode calls, within the
    layer tolerance of the oracle's chain, pad rows zero, and no decode state afterwards."""
    w = wl.WORKLOADS[name]
    cfg, Ws, stack = build(eet, w, n_layers, use_graph=True)
    lens, x = wl.lengths(w), wl.prompt_embeddings(w)
    B = w.batch
    xp = x.copy()
    for b, L in enumerate(lens):
        xp[b, int(L):] = np.nan                      # pad rows are never read
    got = stack.encode(dev(xp), lens)
    layers = [eet.DecoderLayer(cfg, {k: torch.from_numpy(v) for k, v in W.items()}) for W in Ws]
    h, ho = dev(xp), x.astype(np.float64)
    for layer, W in zip(layers, Ws):
        h = layer.encode(h, lens)
        ho = orc.DecoderLayerOracle(W, w.heads, B, w.max_seq, w.ln_eps).encode(ho, lens)
    torch.cuda.synchronize()
    g = host(got)
    assert np.array_equal(g.view(np.uint16), host(h).view(np.uint16))
    for b, L in enumerate(lens):
        L = int(L)
        gate(g[b, :L], ho[b, :L], f"{name} stack encode b={b}")
        assert np.all(g[b, L:] == 0)
    with pytest.raises(eet.EETError) as e:
        stack.decode_step(dev(wl.decode_embeddings(w, 0)))
    assert e.value.code == eet.EET_ERR_STATE
    stack.prefill(dev(x), lens)                      # the stack is usable as a decoder again
    stack.decode_step(dev(wl.decode_embeddings(w, 0)))
    torch.cuda.synchronize()
    assert stack.cache_lens(B) == [int(v) + 1 for v in lens]
    stack.close()
    for layer in layers:
        layer.close()


@pytest.mark.parametrize("use_graph", [False, True])
def test_resume_from_a_saved_cache(eet, use_graph):
    """The resumable state is the K/V cache and the lengths: a second stack (same configuration and weights) that is
    handed a copy of the cache and eet_stack_restore(lengths) continues bit for bit where the first one was, and so does
    a single layer with eet_restore."""
    w = wl.WORKLOADS["small64"]
    cfg, Ws, first = build(eet, w, 2, use_graph=use_graph)
    _, _, second = build(eet, w, 2, use_graph=use_graph)
    lens, x = wl.lengths(w), wl.prompt_embeddings(w)
    B = w.batch
    stream = torch.cuda.Stream()
    steps = [dev(wl.decode_embeddings(w, k)) for k in range(6)]
    with torch.cuda.stream(stream):
        first.prefill(dev(x), lens, stream=stream)
        for k in range(3):
            first.decode_step(steps[k], stream=stream)
    stream.synchronize()
    saved_lens = first.cache_lens(B)
    assert saved_lens == [int(v) + 3 for v in lens]
    second.kv_cache.copy_(first.kv_cache)                               # the checkpoint: cache bytes + lengths
    torch.cuda.synchronize()
    with pytest.raises(eet.EETError) as e:
        second.decode_step(steps[3])
    assert e.value.code == eet.EET_ERR_STATE                            # nothing restored yet
    eet.eet_stack_restore(second.handle, saved_lens, stream=stream)
    with torch.cuda.stream(stream):
        a = [first.decode_step(steps[k], stream=stream) for k in range(3, 6)]
        b = [second.decode_step(steps[k], stream=stream) for k in range(3, 6)]
    stream.synchronize()
    for ya, yb in zip(a, b):
        assert torch.equal(ya, yb)
    assert torch.equal(first.kv_cache, second.kv_cache)
    assert first.cache_lens(B) == second.cache_lens(B) == [int(v) + 6 for v in lens]
    with pytest.raises(eet.EETError) as e:
        eet.eet_stack_restore(second.handle, [w.max_seq + 1] + saved_lens[1:])
    assert e.value.code == eet.EET_ERR_INVALID_ARG
    first.close()
    second.close()
    # one layer
    la = eet.DecoderLayer(cfg, {k: torch.from_numpy(v) for k, v in Ws[0].items()}, cache_fill=SENTINEL)
    lb = eet.DecoderLayer(cfg, {k: torch.from_numpy(v) for k, v in Ws[0].items()}, cache_fill=SENTINEL)
    la.prefill(dev(x), lens)
    la.decode_step(steps[0])
    torch.cuda.synchronize()
    lb.kv_cache.copy_(la.kv_cache)
    eet.eet_restore(lb.handle, la.cache_lens(B))
    ya, yb = la.decode_step(steps[1]), lb.decode_step(steps[1])
    torch.cuda.synchronize()
    assert torch.equal(ya, yb) and torch.equal(la.kv_cache, lb.kv_cache) and la.cache_lens(B) == lb.cache_lens(B)
    la.close()
    lb.close()


class Guarded:
    """A device buffer with a megabyte of 0xA5 on either side: nothing may ever write there."""
    GUARD = 1 << 20

    def __init__(self, nbytes):
        self.nbytes = nbytes
        self.raw = torch.full((nbytes + 2 * self.GUARD,), 0xA5, dtype=torch.uint8, device="cuda:0")
        self.mid = self.raw[self.GUARD: self.GUARD + nbytes]
        assert self.mid.data_ptr() % 256 == 0

    def intact(self):
        return bool((self.raw[: self.GUARD] == 0xA5).all()) and bool((self.raw[self.GUARD + self.nbytes:] == 0xA5).all())


@pytest.mark.parametrize("name,n_layers", [("small64", 2), ("small128", 1), ("wide1280", 2)])
def test_nothing_is_written_outside_the_sizes_the_library_asks_for(eet, name, n_layers):
    """Workspace, K/V cache, model workspace, outputs and logits are handed over with guard regions around exactly the
    number of bytes the size queries name; prefill, decode steps, the encoder pass and the model calls leave every
    guard untouched (and still agree with a run on ordinary buffers)."""
    w = wl.WORKLOADS[name]
    V = 200
    cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
    Ws = [{k: dev(v) for k, v in wl.layer_weights(w, li, random_affine=True).items()} for li in range(n_layers)]
    head = {k: dev(v) for k, v in wl.model_head(w, 256, w.max_seq).items()}           # 256 rows: the padded vocabulary
    mcfg = eet.ModelConfig(V, 256, w.max_seq)
    ws = Guarded(eet.eet_stack_workspace_bytes(cfg, n_layers))
    kv = Guarded(eet.eet_stack_kv_cache_bytes(cfg, n_layers))
    mws = Guarded(eet.eet_model_workspace_bytes(cfg, mcfg))
    lens, x = wl.lengths(w), wl.prompt_embeddings(w)
    B, S, H = x.shape
    out = Guarded(2 * B * S * H)
    dout = Guarded(2 * B * H)
    logits = Guarded(2 * B * 256)
    nxt = Guarded(4 * B)
    stack = eet.eet_stack_create(cfg, Ws, ws.mid, use_graph=True)
    model = eet.eet_model_create(stack, cfg, mcfg, head, mws.mid)
    stream = torch.cuda.Stream()
    ids = dev(np.where(wl.prompt_ids(w, V) < 0, 0, wl.prompt_ids(w, V)).astype(np.int32))
    ref = eet.DecoderStack(cfg, [{k: v for k, v in W.items()} for W in Ws], use_graph=False)
    with torch.cuda.stream(stream):
        eet.eet_stack_prefill(stack, lens, B, S, dev(x), out.mid, kv.mid, stream)
        for k in range(3):
            eet.eet_stack_decode_step(stack, dev(wl.decode_embeddings(w, k)), dout.mid, kv.mid, stream)
    stream.synchronize()
    want = ref.prefill(dev(x), lens)
    for k in range(3):
        want_d = ref.decode_step(dev(wl.decode_embeddings(w, k)))
    torch.cuda.synchronize()
    assert torch.equal(out.mid.view(torch.float16).view(B, S, H), want)
    assert torch.equal(dout.mid.view(torch.float16).view(B, H), want_d)
    with torch.cuda.stream(stream):
        eet.eet_stack_encode(stack, lens, B, S, dev(x), out.mid, kv.mid, stream)
        eet.eet_stack_prefill_left_padded(stack, lens, B, S, dev(x), out.mid, kv.mid, stream)
        eet.eet_model_prefill(model, lens, B, S, ids, logits.mid, nxt.mid, kv.mid, stream)
        for k in range(3):
            eet.eet_model_decode_step(model, nxt.mid.view(torch.int32), logits.mid, nxt.mid, kv.mid, stream)
        eet.eet_model_prefill_left_padded(model, lens, B, S, ids, logits.mid, nxt.mid, kv.mid, stream)
    stream.synchronize()
    for g, what in ((ws, "workspace"), (kv, "K/V cache"), (mws, "model workspace"), (out, "prefill output"), (dout, "decode output"),
                    (logits, "logits"), (nxt, "next ids")):
        assert g.intact(), what
    assert bool(torch.isfinite(logits.mid.view(torch.float16)).all())
    eet.eet_model_destroy(model)
    eet.eet_stack_destroy(stack)
    ref.close()
