"""Model-level parity: eet_op_embedding / eet_op_argmax and eet_model_prefill / eet_model_decode_step through the
C ABI against the CPU oracle.

Integer and table work is compared bit for bit (embedding rows are one exactly-rounded fp16 sum; the greedy choice
is taken by both sides over the same fp16 logits).  The floating-point parts are gated part by part, each fed what
the GPU handed to it (embedding -> the stack -> final LayerNorm + output projection), and end to end on a two-layer
model; the stack itself is covered layer by layer in test_gpu_layer.py.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl
from tests.gpu_util import MAX_ABS, MEAN_ABS, dev, gate, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def fp16_sum(wte, wpe, ids, pos):
    """The oracle's embedding rounded once to fp16 (the sum of two fp16 values is exact in float64)."""
    return orc.embedding(ids, pos, wte, wpe).astype(np.float16)


# ------------------------------------------------------------------------------------------ operators
@pytest.mark.parametrize("H,S,lens", [(256, 40, [40, 1, 17]), (1280, 9, [3, 9]), (8, 5, [5, 2, 1, 4])])
def test_embedding_op_is_bit_exact_and_skips_pad_ids(eet, H, S, lens):
    V, P, B = 1000, 64, len(lens)
    w = wl.Workload("e", 41, H, 1, 64, 1, B, S, 1, S, 0, P)
    head = wl.model_head(w, V, P)
    ids = wl.uniform_int(41, 9, B * S, 0, V - 1).reshape(B, S)
    for b, L in enumerate(lens):
        ids[b, L:] = -7 if b % 2 else 10 ** 9          # pad ids: out of range, must never be read
    out = torch.full((B, S, H), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_embedding(dev(ids), lens, dev(head["wte"]), dev(head["wpe"]), out)
    torch.cuda.synchronize()
    got = host(out)
    for b, L in enumerate(lens):
        want = fp16_sum(head["wte"], head["wpe"], ids[b, :L], range(L))
        assert np.array_equal(got[b, :L].view(np.uint16), want.view(np.uint16)), f"sequence {b}"
        assert np.all(got[b, L:] == 0)


def test_left_padded_embedding_op(eet):
    V, P, H, S, lens = 300, 40, 128, 33, [33, 1, 20, 32]
    B = len(lens)
    w = wl.Workload("e", 45, H, 1, 64, 1, B, S, 1, S, 0, P)
    head = wl.model_head(w, V, P)
    ids = np.full((B, S), -3, np.int32)                              # pad ids in front: out of range, never read
    tok = wl.uniform_int(45, 9, B * S, 0, V - 1).reshape(B, S)
    for b, L in enumerate(lens):
        ids[b, S - L:] = tok[b, :L]
    out = torch.full((B, S, H), float("nan"), dtype=torch.float16, device="cuda:0")
    eet.eet_op_embedding_left_padded(dev(ids), lens, dev(head["wte"]), dev(head["wpe"]), out)
    torch.cuda.synchronize()
    got = host(out)
    for b, L in enumerate(lens):
        want = fp16_sum(head["wte"], head["wpe"], tok[b, :L], range(L))     # token t of the sequence: position t
        assert np.array_equal(got[b, S - L:].view(np.uint16), want.view(np.uint16)), f"sequence {b}"
        assert np.all(got[b, :S - L] == 0)


def test_embedding_rows_with_an_id_or_position_outside_the_tables_become_nan(eet):
    V, P, H, S = 50, 6, 64, 8
    w = wl.Workload("e", 43, H, 1, 64, 1, 2, S, 1, S, 0, P)
    head = wl.model_head(w, V, P)
    ids = wl.uniform_int(43, 9, 2 * S, 0, V - 1).reshape(2, S)
    ids[0, 2], ids[1, 0] = V, -1
    out = torch.zeros((2, S, H), dtype=torch.float16, device="cuda:0")
    eet.eet_op_embedding(dev(ids), [8, 5], dev(head["wte"]), dev(head["wpe"]), out)     # positions 6, 7 of sequence 0 >= max_pos
    torch.cuda.synchronize()
    got = host(out)
    bad = {(0, 2), (0, 6), (0, 7), (1, 0)}
    for b, L in enumerate([8, 5]):
        for i in range(L):
            if (b, i) in bad:
                assert np.all(np.isnan(got[b, i]))
            else:
                assert np.array_equal(got[b, i], fp16_sum(head["wte"], head["wpe"], [ids[b, i]], [i])[0])
    # decode form: positions come from the device
    tok = np.array([3, V, 7, 0], np.int32); pos = np.array([5, 0, 6, -1], np.int32)
    o2 = torch.zeros((4, H), dtype=torch.float16, device="cuda:0")
    eet.eet_op_embedding_decode(dev(tok), dev(pos), dev(head["wte"]), dev(head["wpe"]), o2)
    torch.cuda.synchronize()
    g2 = host(o2)
    assert np.array_equal(g2[0], fp16_sum(head["wte"], head["wpe"], [3], [5])[0])
    assert np.all(np.isnan(g2[1:]))


@pytest.mark.parametrize("V,stride", [(50257, 50304), (5, 8), (13, 16), (2048, 2048), (777, 1024)])
def test_argmax_op_takes_the_first_maximum_of_the_valid_columns(eet, V, stride):
    rows = 9
    lg = wl.normal(47, V, (rows, stride), 2.0)
    lg[:, V:] = 60000.0                                   # padding columns hold the largest values
    lg[1, :] = lg[1, 0]                                   # all equal: index 0
    top = np.float16(lg[2, :V].astype(np.float32).max())
    lg[2, V - 1] = top                                    # the maximum again in the last valid column: the earlier one wins
    lg[3, :V] = -np.inf                                   # nothing above -inf: 0
    lg[4, ::3] = np.nan                                   # NaN never wins
    lg[5, V // 2] = 30000.0
    lg[6, V - 1] = 30000.0                                # the tail of the row
    lg[7, 0] = 30000.0
    out = torch.full((rows,), -1, dtype=torch.int32, device="cuda:0")
    eet.eet_op_argmax(dev(lg), out, vocab=V)
    torch.cuda.synchronize()
    want = orc.greedy_token(lg.astype(np.float64), V)
    assert host(out).tolist() == want.tolist()
    assert want[1] == 0 and want[3] == 0 and want[5] == V // 2 and want[6] == V - 1 and want[7] == 0


# ------------------------------------------------------------------------------------------ the model
def build(eet, w, vocab, affine=True, use_graph=True):
    LW = [wl.layer_weights(w, l, random_affine=affine) for l in range(w.layers)]
    head = wl.model_head(w, vocab, w.max_seq, random_affine=affine)
    cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
    gpu = eet.DecoderModel(cfg, [{k: torch.from_numpy(v) for k, v in W.items()} for W in LW],
                           {k: torch.from_numpy(v) for k, v in head.items()}, vocab, use_graph=use_graph)
    head = {k: v.astype(np.float64) for k, v in head.items()}       # widened once (exactly) for the oracle's functions
    ora = orc.DecoderModelOracle(LW, head, w.heads, w.batch, w.max_seq, w.ln_eps)
    return gpu, ora, head


def check_head(gpu, head, hidden_rows, logits, nxt, vocab, what):
    """Final LayerNorm + output projection fed the GPU's own last-layer rows; greedy choice over the GPU's own logits."""
    lg = host(logits)
    want = orc.lm_head(hidden_rows.astype(np.float64), head["lnf_g"], head["lnf_b"], head["wte"])
    gate(lg[:, :vocab], want, f"{what}: logits from the GPU's hidden rows")
    assert host(nxt).tolist() == orc.greedy_token(lg.astype(np.float64), vocab).tolist(), f"{what}: greedy choice"
    return lg


@pytest.mark.parametrize("use_graph", [True, False])
def test_small_model_part_by_part_and_end_to_end(eet, use_graph):
    w = replace(wl.WORKLOADS["small64"], decode_steps=4)           # 2 layers, hidden 256, 5 ragged prompts of 3..200 tokens
    V = 1000
    gpu, ora, head = build(eet, w, V, use_graph=use_graph)
    lens = [int(v) for v in wl.lengths(w)]
    ids = wl.prompt_ids(w, V, pad_value=-1)
    B, S = ids.shape
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        logits, nxt = gpu.prefill(dev(ids), lens, stream=stream)
    stream.synchronize()
    want = ora.prefill(ids, lens)
    h_in, h_out = gpu.hidden_states(decode=False)
    assert h_in is None                   # two layers: the final output sits where the embedding was (Section 3.1, first rule)
    h_out = host(h_out)
    for b, L in enumerate(lens):
        assert np.all(h_out[b, L:] == 0)
        gate(h_out[b, :L], ora.hidden_out[b, :L], f"two free-running layers b={b}", 2 * MAX_ABS, 2 * MEAN_ABS)
    last = np.stack([h_out[b, L - 1] for b, L in enumerate(lens)])
    lg = check_head(gpu, head, last, logits, nxt, V, "prefill")
    gate(lg[:, :V], want, "prefill: logits end to end")
    assert np.all(lg[:, V:] == 0)                                   # rows of wte beyond the vocabulary are zero here
    assert gpu.stack.cache_lens(B) == lens
    for k in range(w.decode_steps):
        step_ids = wl.decode_ids(w, k, V)
        with torch.cuda.stream(stream):
            logits, nxt = gpu.decode_step(dev(step_ids), stream=stream)
        stream.synchronize()
        want = ora.decode_step(step_ids)
        d_in, d_out = [host(t) for t in gpu.hidden_states(decode=True)]
        assert np.array_equal(d_in.view(np.uint16), fp16_sum(head["wte"], head["wpe"], step_ids, [L + k for L in lens]).view(np.uint16))
        lg = check_head(gpu, head, d_out, logits, nxt, V, f"decode {k}")
        gate(lg[:, :V], want, f"decode {k}: logits end to end")
        assert gpu.stack.cache_lens(B) == [L + k + 1 for L in lens]
    gpu.close()


def test_generation_feeds_the_chosen_tokens_back_on_the_device(eet):
    """Greedy generation with no host round trip: the ids of step k+1 are the next_ids buffer of step k.  The oracle is
    fed the tokens the GPU chose; the two choices must agree wherever the oracle's best logit leads by more than the
    tolerance on a logit (both sides of a closer call are correct)."""
    w = replace(wl.WORKLOADS["small64"], batch=3, decode_steps=8)
    V = 520                                                         # padded to 576: several padding columns
    gpu, ora, head = build(eet, w, V)
    lens = [int(v) for v in wl.lengths(w)]
    ids = wl.prompt_ids(w, V)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        logits, nxt = gpu.prefill(dev(ids), lens, stream=stream)
        steps = [(logits, nxt)]
        for k in range(w.decode_steps):
            logits, nxt = gpu.decode_step(nxt, stream=stream)        # device to device
            steps.append((logits, nxt))
    stream.synchronize()
    want = ora.prefill(ids, lens)
    agree = total = 0
    for k, (logits, nxt) in enumerate(steps):
        lg, chosen = host(logits), host(nxt)
        gate(lg[:, :V], want, f"generation step {k}: logits")
        assert chosen.tolist() == orc.greedy_token(lg.astype(np.float64), V).tolist()
        assert np.all((0 <= chosen) & (chosen < V))
        srt = np.sort(want, axis=1)
        clear = srt[:, -1] - srt[:, -2] > 2 * MAX_ABS
        assert np.array_equal(chosen[clear], orc.greedy_token(want)[clear])
        agree += int((chosen == orc.greedy_token(want)).sum()); total += len(chosen)
        if k < w.decode_steps:
            want = ora.decode_step(chosen)
    assert gpu.stack.cache_lens(w.batch) == [L + w.decode_steps for L in lens]
    print(f"\n[generation] GPU and oracle chose the same token in {agree} of {total} steps")
    gpu.close()


@pytest.mark.parametrize("layers", [1, 2])
def test_left_padded_model_prefill(eet, layers):
    """Pads in front: logits, greedy tokens, caches and lengths are bit for bit those of the right-padded call on the same
    tokens (and so within tolerance of the oracle's left-padded model), and generation continues identically."""
    w = replace(wl.WORKLOADS["small64"], layers=layers, decode_steps=2)
    V = 1000
    right, ora, head = build(eet, w, V)
    left, _, _ = build(eet, w, V)
    lens = [int(v) for v in wl.lengths(w)]
    ids = wl.prompt_ids(w, V, pad_value=-1)
    B, S = ids.shape
    ids_l = np.full_like(ids, -1)
    for b, L in enumerate(lens):
        ids_l[b, S - L:] = ids[b, :L]
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lr, nr = right.prefill(dev(ids), lens, stream=stream)
        ll, nl = left.prefill(dev(ids_l), lens, stream=stream, left_padded=True)
    stream.synchronize()
    assert np.array_equal(host(ll).view(np.uint16), host(lr).view(np.uint16)) and host(nl).tolist() == host(nr).tolist()
    gate(host(ll)[:, :V], ora.prefill(ids_l, lens, left_padded=True), "left-padded model: logits")
    h_in, h_out = left.hidden_states(decode=False)
    if layers % 2:                                                    # the embedding is still in its activation cache
        for b, L in enumerate(lens):
            assert np.array_equal(host(h_in)[b, S - L:].view(np.uint16),
                                  fp16_sum(head["wte"], head["wpe"], ids[b, :L], range(L)).view(np.uint16))
            assert np.all(host(h_in)[b, :S - L] == 0)
    else:
        assert h_in is None
    for b, L in enumerate(lens):
        assert np.all(host(h_out)[b, :S - L] == 0)
    assert torch.equal(left.stack.kv_cache, right.stack.kv_cache)
    assert left.stack.cache_lens(B) == right.stack.cache_lens(B) == lens
    with torch.cuda.stream(stream):
        for _ in range(w.decode_steps):
            lr, nr = right.decode_step(nr, stream=stream)
            ll, nl = left.decode_step(nl, stream=stream)
    stream.synchronize()
    assert np.array_equal(host(ll).view(np.uint16), host(lr).view(np.uint16)) and host(nl).tolist() == host(nr).tolist()
    left.close()
    right.close()


def test_model_errors_and_poisoned_ids(eet):
    w = replace(wl.WORKLOADS["tiny"], decode_steps=2)               # hidden 64, one head, max_seq 32, prompts padded to 24
    V = 100
    gpu, ora, head = build(eet, w, V)
    lens = [24, 1, 7]
    ids = wl.prompt_ids(w, V)
    ids = np.where(ids < 0, 0, ids).astype(np.int32)
    with pytest.raises(eet.EETError) as e:
        gpu.decode_step(dev(np.zeros(3, np.int32)))
    assert e.value.code == eet.EET_ERR_STATE
    with pytest.raises(eet.EETError) as e:
        gpu.prefill(dev(ids), [24, 0, 7])
    assert e.value.code == eet.EET_ERR_INVALID_ARG
    bad = ids.copy()
    bad[1, 0] = V + 3                                                # inside the padded table, outside the vocabulary
    logits, nxt = gpu.prefill(dev(bad), lens)
    torch.cuda.synchronize()
    lg = host(logits)
    assert np.all(np.isnan(lg[1])) and host(nxt)[1] == 0             # the poisoned sequence is loud ...
    want = ora.prefill(ids, lens)
    gate(lg[[0, 2], :V], want[[0, 2]], "sequences beside a poisoned one")   # ... and the others do not notice
    for k in range(32 - 24):
        gpu.decode_step(dev(np.full(3, k, np.int32)))
    with pytest.raises(eet.EETError) as e:                           # sequence 0 now fills its 32 slots
        gpu.decode_step(dev(np.zeros(3, np.int32)))
    assert e.value.code == eet.EET_ERR_CAPACITY
    torch.cuda.synchronize()
    assert gpu.stack.cache_lens(3) == [32, 9, 15]
    gpu.close()


def test_gpt2_sized_vocabulary_on_the_cfg2_layer_shape(eet):
    """Hidden 1024, 16 heads, batch 8, prompts of 256-512 tokens (the benchmark's layer shape, one layer) with GPT-2's
    vocabulary of 50257 padded to 50304 columns: embedding bit for bit on every valid row, the output projection on all
    50257 logits of every sequence from the GPU's own hidden rows, greedy choice exact; prefill and two decode steps."""
    w = replace(wl.WORKLOADS["cfg2"], layers=1, decode_steps=2)
    V = 50257
    gpu, ora, head = build(eet, w, V, affine=False)
    lens = [int(v) for v in wl.lengths(w)]
    ids = wl.prompt_ids(w, V)
    B, S = ids.shape
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        logits, nxt = gpu.prefill(dev(ids), lens, stream=stream)
    stream.synchronize()
    h_in, h_out = [host(t) for t in gpu.hidden_states(decode=False)]
    for b, L in enumerate(lens):
        assert np.array_equal(h_in[b, :L].view(np.uint16), fp16_sum(head["wte"], head["wpe"], ids[b, :L], range(L)).view(np.uint16))
        assert np.all(h_in[b, L:] == 0)
    # the layer between the two, on the last valid row of every sequence (the row the logits are taken from)
    layer = ora.layers[0]
    x = np.zeros((B, S, w.hidden))
    for b, L in enumerate(lens):
        x[b, :L] = h_in[b, :L]
    ref = layer.prefill(x, lens, rows={b: [L - 1] for b, L in enumerate(lens)})
    last = np.stack([h_out[b, L - 1] for b, L in enumerate(lens)])
    gate(last, np.stack([ref[b, L - 1] for b, L in enumerate(lens)]), "cfg2-shape layer, last rows")
    check_head(gpu, head, last, logits, nxt, V, "cfg2-shape prefill")
    for k in range(w.decode_steps):
        with torch.cuda.stream(stream):
            logits, nxt2 = gpu.decode_step(nxt, stream=stream)
        stream.synchronize()
        fed = host(nxt)
        d_in, d_out = [host(t) for t in gpu.hidden_states(decode=True)]
        assert np.array_equal(d_in.view(np.uint16), fp16_sum(head["wte"], head["wpe"], fed, [L + k for L in lens]).view(np.uint16))
        gate(d_out, layer.decode_step(d_in.astype(np.float64)), f"cfg2-shape layer, decode {k}")
        check_head(gpu, head, d_out, logits, nxt2, V, f"cfg2-shape decode {k}")
        nxt = nxt2
    assert gpu.stack.cache_lens(B) == [L + w.decode_steps for L in lens]
    gpu.close()


def differs(what, a, b):
    """Message for a failed bit-for-bit comparison: how many elements differ, where the first one is, by how much."""
    a, b = a.reshape(-1), b.reshape(-1)
    ne = (a != b) & ~(torch.isnan(a.float()) & torch.isnan(b.float()))
    idx = torch.nonzero(ne).reshape(-1)
    if idx.numel() == 0:
        return f"{what}: NaN patterns differ"
    i = int(idx[0])
    return (f"{what}: {idx.numel()} of {a.numel()} elements differ, first at flat index {i} ({float(a[i])} vs {float(b[i])}), "
            f"largest difference {float((a.float() - b.float()).abs()[idx].max())}")


def test_cfg2_model_at_full_size_is_embedding_then_stack_then_head(eet):
    """The benchmark's --model configuration (24 layers, batch 8, prompts of 256-512 tokens, vocabulary 50257, decode
    steps replayed from the stack's graph): the model call is bit for bit the embedding operator, then the stack entry
    points on a second stack with the same weights, and its logits are the output projection of its own last-layer rows
    within tolerance, with the exact greedy choice -- each of those parts is compared with the oracle on its own
    (embedding: above; stack: layer by layer in test_gpu_layer.py; head: check_head)."""
    w = replace(wl.WORKLOADS["cfg2"], decode_steps=3)
    V = 50257
    LW = [{k: torch.from_numpy(v) for k, v in wl.layer_weights(w, l).items()} for l in range(w.layers)]
    head = wl.model_head(w, V, w.max_seq)
    cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
    model = eet.DecoderModel(cfg, LW, {k: torch.from_numpy(v) for k, v in head.items()}, V)
    other = eet.DecoderStack(cfg, LW, use_graph=False)
    head64 = {k: v.astype(np.float64) for k, v in head.items()}
    lens = [int(v) for v in wl.lengths(w)]
    ids = dev(wl.prompt_ids(w, V))
    B, S = ids.shape
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        logits, nxt = model.prefill(ids, lens, stream=stream)
    stream.synchronize()
    h_in, h_out = model.hidden_states(decode=False)
    assert h_in is None                                             # 24 layers: the final output replaced the embedding
    emb = torch.empty((B, S, w.hidden), dtype=torch.float16, device="cuda:0")
    eet.eet_op_embedding(ids, lens, model.head["wte"], model.head["wpe"], emb, vocab=V)
    ref = other.prefill(emb, lens)
    torch.cuda.synchronize()
    assert torch.equal(h_out, ref), differs("prefill: last-layer rows, model against embedding operator + stack", h_out, ref)
    last = np.stack([host(h_out[b, L - 1]) for b, L in enumerate(lens)])
    check_head(model, head64, last, logits, nxt, V, "cfg2 model prefill")
    for k in range(w.decode_steps):
        fed = nxt
        with torch.cuda.stream(stream):
            logits, nxt = model.decode_step(fed, stream=stream)
        stream.synchronize()
        d_in, d_out = model.hidden_states(decode=True)
        pos = torch.tensor([L + k for L in lens], dtype=torch.int32, device="cuda:0")
        x = torch.empty((B, w.hidden), dtype=torch.float16, device="cuda:0")
        eet.eet_op_embedding_decode(fed, pos, model.head["wte"], model.head["wpe"], x, vocab=V)
        y = other.decode_step(x)
        torch.cuda.synchronize()
        assert torch.equal(d_in, x), differs(f"decode {k}: embedded rows", d_in, x)
        assert torch.equal(d_out, y), differs(f"decode {k}: last-layer rows", d_out, y)
        check_head(model, head64, host(d_out), logits, nxt, V, f"cfg2 model decode {k}")
    assert model.stack.cache_lens(B) == other.cache_lens(B) == [L + w.decode_steps for L in lens]
    assert torch.equal(model.stack.kv_cache, other.kv_cache), differs("K/V caches", model.stack.kv_cache, other.kv_cache)
    model.close()
    other.close()


def test_model_sized_for_more_sequences_serves_smaller_batches_one_after_another(eet):
    """A model created for 6 sequences runs a batch of 4, generates, then a batch of 2 with other prompts, generates again
    (the recorded decode graph is re-recorded for the new batch): every call against a fresh oracle model."""
    w = replace(wl.WORKLOADS["small64"], batch=6, decode_steps=3)
    V = 333
    gpu, _, head = build(eet, w, V)
    LW = [wl.layer_weights(w, l, random_affine=True) for l in range(w.layers)]
    all_ids = wl.prompt_ids(w, V)
    all_lens = [int(v) for v in wl.lengths(w)]
    stream = torch.cuda.Stream()
    for rows in ([0, 1, 2, 3], [5, 4]):
        ids = np.ascontiguousarray(all_ids[rows]); lens = [all_lens[r] for r in rows]
        ora = orc.DecoderModelOracle(LW, head, w.heads, len(rows), w.max_seq, w.ln_eps)
        with torch.cuda.stream(stream):
            logits, nxt = gpu.prefill(dev(ids), lens, stream=stream)
        stream.synchronize()
        want = ora.prefill(ids, lens)
        gate(host(logits)[:, :V], want, f"batch of {len(rows)}: prefill logits")
        for k in range(w.decode_steps):
            fed = host(nxt)
            with torch.cuda.stream(stream):
                logits, nxt = gpu.decode_step(nxt, stream=stream)
            stream.synchronize()
            want = ora.decode_step(fed)
            gate(host(logits)[:, :V], want, f"batch of {len(rows)}: decode {k} logits")
            assert host(nxt).tolist() == orc.greedy_token(host(logits).astype(np.float64), V).tolist()
        assert gpu.stack.cache_lens(len(rows)) == [L + w.decode_steps for L in lens]
    gpu.close()
