#!/usr/bin/env python3
"""Benchmark of the decoder-layer hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch of the named workload:
whole-prompt prefill through every layer, then every incremental decode step through every
layer (K/V caches filled by the prefill and extended by each step).  Inputs, weights and caches
are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5b] [--also cfg2,cfg3,cfg4,cfg5a]

The line's metric, value and roofline are those of --workload (default: cfg5b, the largest configuration, where the
60 % HBM / 50 % MFMA targets are defined); the workloads of --also are timed the same way, with fewer passes, and
reported under "other_workloads" in the same line, each with its own roofline records.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_FP16_PEAK_TFLOPS = 2500.0  # dense fp16 MFMA, published

PROFILES = os.path.join(ROOT, "profiles")


def profiled_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 hardware counters (two --pmc runs, FETCH_SIZE and WRITE_SIZE, each
    scaled by what the same counter reads for a plain copy of known size), read from the committed summary
    profiles/<workload>_hbm_traffic_counters.txt: lines of the form
        traffic | <start of the record's kernel name> | <bytes per launch>
    and one line `measured: <commit, date, command>`.  Returns ({prefix: bytes}, source string); workloads without a
    summary report null.  Nothing here is measured by this run: the record says where the figure comes from."""
    path = os.path.join(PROFILES, f"{workload}_hbm_traffic_counters.txt")
    table, measured = {}, ""
    if os.path.exists(path):
        for line in open(path):
            parts = [t.strip() for t in line.split("|")]
            if len(parts) == 3 and parts[0] == "traffic":
                try:
                    table[parts[1]] = float(parts[2])
                except ValueError:
                    pass
            elif line.startswith("measured:"):
                measured = line[len("measured:"):].strip()
    return table, (f"profiles/{os.path.basename(path)}" + (f" ({measured})" if measured else "")) if table else None


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=3)
    p.add_argument("--warmup", type=int, default=1)
    p.add_argument("--workload", default="cfg5b")
    p.add_argument("--also", default="cfg2,cfg3,cfg4,cfg5a",
                   help="comma-separated workloads reported under other_workloads (two timed passes each); '' for none")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--model", action="store_true",
                   help="run the pass through the model entry points (embedding, the stack, final LayerNorm, output "
                        "projection over GPT-2's vocabulary, greedy choice fed back on the device) instead of the stack's")
    p.add_argument("--no-graph", action="store_true", help="launch decode kernels directly instead of replaying a graph")
    p.add_argument("--kernel-reps", type=int, default=200, help="launches per kernel in the roofline measurement")
    p.add_argument("--roofline-only", action="store_true",
                   help="skip the timed pass and the CPU baseline: only the per-kernel measurement plus one plain "
                        "256 MiB device copy (the reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    return p.parse_args()


class Stack:
    """The workload's layers behind the stack entry points (one call per prefill, one per decode
    step; decode steps are replayed from a HIP graph recorded by the library), on its own stream."""

    def __init__(self, w, eet, torch, wl, use_graph=True, device_weights=None):
        self.w, self.eet, self.torch = w, eet, torch
        cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
        if device_weights is None:        # fp16 weights of every layer, uploaded once
            device_weights = [{k: torch.from_numpy(v).to("cuda:0") for k, v in wl.layer_weights(w, li).items()}
                              for li in range(w.layers)]
        self.stack = eet.DecoderStack(cfg, device_weights, use_graph=use_graph)
        self.n_layers = w.layers
        self.lens = [int(v) for v in wl.lengths(w)]
        dev = "cuda:0"
        self.x0 = torch.from_numpy(wl.prompt_embeddings(w)).to(dev)
        self.dec_in = torch.stack([torch.from_numpy(wl.decode_embeddings(w, k)) for k in range(w.decode_steps)]).to(dev) \
            if w.decode_steps else None
        self.pout = torch.empty_like(self.x0)
        self.tok = torch.empty((w.batch, w.hidden), dtype=torch.float16, device=dev)   # fixed decode input buffer
        self.dout = torch.empty_like(self.tok)
        self.stream = torch.cuda.Stream()      # the null stream cannot be captured into a graph

    def weights(self, layer):
        return self.stack.weights[layer]

    def cache_views(self, layer):
        return self.stack.cache_views(layer)

    def prefill(self):
        with self.torch.cuda.stream(self.stream):
            self.stack.prefill(self.x0, self.lens, self.pout)

    def decode(self):
        with self.torch.cuda.stream(self.stream):
            for k in range(self.w.decode_steps):
                self.tok.copy_(self.dec_in[k])          # this step's input embeddings
                self.stack.decode_step(self.tok, self.dout)

    def one_pass(self):
        self.prefill()
        self.decode()


class ModelStack(Stack):
    """The same layers behind the model entry points at GPT-2's vocabulary: token ids in, one call per prefill and one
    per decode step, the greedy token of a step fed to the next step on the device (no host round trip)."""
    VOCAB = 50257

    def __init__(self, w, eet, torch, wl, use_graph=True):
        self.w, self.eet, self.torch = w, eet, torch
        cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
        weights = [{k: torch.from_numpy(v) for k, v in wl.layer_weights(w, li).items()} for li in range(w.layers)]
        head = {k: torch.from_numpy(v) for k, v in wl.model_head(w, self.VOCAB, w.max_seq).items()}
        self.model = eet.DecoderModel(cfg, weights, head, self.VOCAB, use_graph=use_graph)
        self.stack = self.model.stack
        self.n_layers = w.layers
        self.lens = [int(v) for v in wl.lengths(w)]
        self.ids = torch.from_numpy(wl.prompt_ids(w, self.VOCAB)).to("cuda:0")
        self.stream = torch.cuda.Stream()
        self.nxt = None

    def prefill(self):
        with self.torch.cuda.stream(self.stream):
            _, self.nxt = self.model.prefill(self.ids, self.lens, stream=self.stream)

    def decode(self):
        with self.torch.cuda.stream(self.stream):
            nxt = self.nxt
            for _ in range(self.w.decode_steps):
                _, nxt = self.model.decode_step(nxt, stream=self.stream)


class EncoderStack:
    """The workload's layers used as a bidirectional encoder (no sequence mask, no decode): one eet_stack_encode call
    per pass, activations in the stack's two activation caches, one layer's K/V region as the scratch of every layer."""

    def __init__(self, w, eet, torch, wl):
        self.w, self.eet, self.torch = w, eet, torch
        cfg = eet.make_config(w.hidden, w.heads, w.ffn, w.batch, w.padded_len, w.max_seq, w.ln_eps)
        self.stack = eet.DecoderStack(cfg, [{k: torch.from_numpy(v) for k, v in wl.layer_weights(w, li).items()}
                                            for li in range(w.layers)], use_graph=False)
        self.n_layers = w.layers
        self.lens = [int(v) for v in wl.lengths(w)]
        self.x0 = torch.from_numpy(wl.prompt_embeddings(w)).to("cuda:0")
        self.out = torch.empty_like(self.x0)
        self.stream = torch.cuda.Stream()

    def weights(self, layer):
        return self.stack.weights[layer]

    def cache_views(self, layer):
        return self.stack.cache_views(layer)

    def prefill(self):
        with self.torch.cuda.stream(self.stream):
            self.stack.encode(self.x0, self.lens, self.out)

    def decode(self):
        pass

    def one_pass(self):
        self.prefill()


def time_region(torch, fn, reps, stream=None):
    """Average duration of fn() in ms, HIP events on the stream the kernels are launched on."""
    s = stream if stream is not None else torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(s)
    for _ in range(reps):
        fn()
    e1.record(s)
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def time_launches(torch, fn, calls, replays=5):
    """Average duration of one fn() in ms with the launches truly back to back: `calls` invocations
    are captured into a HIP graph on the launch stream (the library only enqueues kernels, so a
    capture records exactly its launches) and the graph is replayed between two HIP events.  A
    Python loop cannot issue launches as fast as these kernels run."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(calls):
            fn()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(calls):
            fn()
    g.replay()
    torch.cuda.synchronize()
    s = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(s)
    for _ in range(replays):
        g.replay()
    e1.record(s)
    e1.synchronize()
    return e0.elapsed_time(e1) / (replays * calls)


def _kernel_candidates(stack, torch, eet, reps, full=True):
    """Time the kernels that can dominate a pass, each through its operator-level entry point on
    the stack's own weights and caches, cycling over the layers so that nothing is served from a
    cache the real pass would not have.  Returns a list of records with the algorithmic bytes or
    flops of one launch, the average launch duration and the launches per pass.  full = False leaves
    out the operators that are not on the layer's path (stand-alone softmax, add-bias kernels, model head)."""
    w = stack.w
    B, H, F, nl = w.batch, w.hidden, w.ffn, stack.n_layers
    d = H // w.heads
    T = sum(stack.lens)
    out = []
    # What a decode step of the real pass moves between two uses of the same operand: every layer's weights and visible
    # K/V once.  An operator-level launch that cycled over less than that (one layer whose output projection is 300 MB,
    # replayed back to back) would find its operand in the 256 MB memory-side cache, which the pass does not: such
    # records cycle over copies of their operand until the cycle is as large as the pass's (capped at 2 GB).
    step_bytes = nl * (2.0 * (4 * H * H + 2 * H * F) + 4.0 * H * sum(L + w.decode_steps // 2 for L in stack.lens))

    def n_copies(bytes_per_launch):
        want = min(step_bytes, 2.0e9)
        return max(1, int(-(-want // (nl * bytes_per_launch))))
    if w.decode_steps:
        # (1) decode attention: K and V of every visible slot read once, q read, ctx written
        ks = sorted({0, w.decode_steps // 4, w.decode_steps // 2, 3 * w.decode_steps // 4, w.decode_steps - 1})
        nkeys = [torch.tensor([L + k + 1 for L in stack.lens], dtype=torch.int32, device="cuda:0") for k in ks]
        bytes_k = [4.0 * H * sum(L + k + 1 for L in stack.lens) + 4.0 * B * H for k in ks]
        scratch = torch.empty(eet.eet_op_attention_decode_scratch_bytes(B, w.heads, d, w.max_seq), dtype=torch.uint8,
                              device="cuda:0")
        q = torch.randn(B, H, device="cuda:0").half()
        ctx = torch.empty_like(q)
        st = {"i": 0}

        caches = [stack.cache_views(i) for i in range(nl)]
        for _ in range(n_copies(sum(bytes_k) / len(bytes_k)) - 1):
            caches += [(kc.clone(), vc.clone()) for kc, vc in caches[:nl]]

        def run_attn():
            i = st["i"]
            st["i"] += 1
            kc, vc = caches[i % len(caches)]
            eet.eet_op_attention_decode(q, kc, vc, ctx, nkeys[(i // len(caches)) % len(ks)], scratch)
        n = len(caches) * len(ks)
        ms = time_launches(torch, run_attn, n * max(1, reps // n))
        out.append({"kernel": f"attn_decode<{d}, 4> (+ attn_decode_combine when the key range is split): decode attention over the K/V cache",
                    "bound": "hbm", "work": sum(bytes_k) / len(bytes_k), "ms": ms,
                    "launches": w.decode_steps * nl})
        del caches
        # (2) decode projections (weight stream) that have an operator-level twin: FFN-2 + bias +
        # residual and the attention output projection + bias + residual.  (The QKV and FFN-1
        # launches of small layers carry a fused LayerNorm and exist only inside the layer call.)
        def projection(name, wkey, bkey, n_out, n_in):
            x = torch.randn(B, n_in, device="cuda:0").half()
            r = torch.randn(B, n_out, device="cuda:0").half()
            y = torch.empty(B, n_out, device="cuda:0", dtype=torch.float16)
            st2 = {"i": 0}
            mats = [(stack.weights(i)[wkey], stack.weights(i)[bkey]) for i in range(nl)]
            for _ in range(n_copies(2.0 * n_out * n_in) - 1):
                mats += [(m.clone(), b_) for m, b_ in mats[:nl]]

            def run():
                m, b_ = mats[st2["i"] % len(mats)]
                st2["i"] += 1
                eet.eet_op_linear(x, m, b_, y, residual=r)
            ms = time_launches(torch, run, len(mats) * max(1, reps // len(mats)))
            out.append({"kernel": f"decode {name} + bias + residual (weight stream, M = {B} rows)", "bound": "hbm",
                        "work": 2.0 * (n_out * n_in + B * n_in + n_out + 2 * B * n_out), "ms": ms,
                        "launches": w.decode_steps * nl})
        projection("FFN-2 projection", "w_fc2", "b_fc2", H, F)
        projection("attention output projection", "w_o", "b_o", H, H)
    # (3) prefill projections on the matrix cores, all valid tokens: the four shapes of a layer (the QKV shape through
    # the plain-bias epilogue: the cache scatter exists only inside the layer call)
    xp = torch.randn(T, H, device="cuda:0").half()
    # the layer keeps the rows of its feed-forward buffer 128 bytes further apart than their length when they are 64 KB or
    # longer (eet_op_linear_strided in include/eet.h); the records of the two feed-forward projections use that layout
    ffn_stride = F + 64 if F >= 32768 else F
    yp = torch.empty(T, ffn_stride, device="cuda:0", dtype=torch.float16)[:, :F]
    yq = torch.empty(T, 3 * H, device="cuda:0", dtype=torch.float16)
    yh = torch.empty(T, H, device="cuda:0", dtype=torch.float16)
    rh = torch.randn(T, H, device="cuda:0").half()
    st3 = {"i": 0}

    def prefill_projection(name, wkey, bkey, x, y, n_out, n_in, act=0, residual=None):
        # a pass uses each weight matrix of a prefill once, with a whole decode phase before its next use: the record
        # cycles over copies (1 GB of them) so that the matrix comes from HBM here too
        mats = [(stack.weights(i)[wkey], stack.weights(i)[bkey]) for i in range(nl)]
        for _ in range(max(1, int(-(-1.0e9 // (nl * 2.0 * n_out * n_in)))) - 1):
            mats += [(m.clone(), b_) for m, b_ in mats[:nl]]

        def run():
            m, b_ = mats[st3["i"] % len(mats)]
            st3["i"] += 1
            (eet.eet_op_linear if x.is_contiguous() and y.is_contiguous() else eet.eet_op_linear_strided)(
                x, m, b_, y, residual=residual, act=act)
        ms = time_launches(torch, run, max(4, min(reps, 24), len(mats)), replays=2)
        # one operator call: one launch of the tile kernel, or two where the library cuts the rows into whole rounds of
        # large tiles plus a small-tile rest (the duration is the call's, the kernel trace lists the two launches)
        out.append({"kernel": f"prefill {name} (MFMA tile kernel, {T} x {n_out} x {n_in})", "bound": "mfma",
                    "work": 2.0 * T * n_out * n_in, "ms": ms, "launches": nl})
    prefill_projection("FFN-1 projection + bias + GELU", "w_fc1", "b_fc1", xp, yp, F, H, act=1)
    yp.normal_()                                    # FFN-2 reads what FFN-1 wrote: keep it finite and O(1)
    prefill_projection("FFN-2 projection + bias + residual", "w_fc2", "b_fc2", yp, yh, H, F, residual=rh)
    prefill_projection("QKV-shaped projection + bias", "w_qkv", "b_qkv", xp, yq, 3 * H, H)
    prefill_projection("attention output projection + bias + residual", "w_o", "b_o", xp, yh, H, H, residual=rh)
    del yq
    # (4) prefill attention: QK^T and PV over the valid causal triangle of every sequence
    qp = torch.randn(B, w.padded_len, H, device="cuda:0").half()
    cp = torch.empty_like(qp)
    st4 = {"i": 0}

    attn_op = eet.eet_op_attention_encoder if w.encoder else eet.eet_op_attention_prefill

    def run_pattn():
        kc, vc = stack.cache_views(st4["i"] % nl)
        st4["i"] += 1
        attn_op(qp, kc, vc, cp, stack.lens, w.heads)
    ms = time_launches(torch, run_pattn, max(4, min(reps, 24)), replays=2)
    pname = "attn_prefill_wide" if d == 128 and max(stack.lens) > 512 else "attn_prefill"      # the library's own choice
    if w.encoder:       # every valid row sees all L valid keys: 2 * (2 * L * L * H) flop per sequence
        out.append({"kernel": f"{pname}<{d}, false>: padding-skipping attention without sequence mask (matrix cores)",
                    "bound": "mfma", "work": sum(4.0 * H * L * L for L in stack.lens), "ms": ms, "launches": nl})
    else:
        out.append({"kernel": f"{pname}<{d}, true>: causal, padding-skipping prefill attention (matrix cores)",
                    "bound": "mfma", "work": sum(2.0 * H * L * (L + 1) for L in stack.lens), "ms": ms, "launches": nl})
    # (5) LayerNorm over the valid rows of the prompt (row kernel, HBM bound): read + write of every row
    xl = torch.randn(T, H, device="cuda:0").half()
    yl = torch.empty_like(xl)
    gam, bet = torch.ones(H, device="cuda:0").half(), torch.zeros(H, device="cuda:0").half()
    ms = time_launches(torch, lambda: eet.eet_op_layernorm(xl, gam, bet, yl, w.ln_eps), max(8, min(reps, 48)), replays=2)
    lname = "layernorm_wave" if H % 8 == 0 and H <= 2048 and T >= 64 else "layernorm_cached"      # the library's own choice
    out.append({"kernel": f"{lname}: LayerNorm over the valid prompt rows (row kernel)", "bound": "hbm",
                "work": 4.0 * T * H + 4.0 * H, "ms": ms, "launches": 2 * nl})
    if not full:
        return out
    # (6) stand-alone mask-free softmax (Algorithm 1) over [B, heads', S, S] scores, in place: the valid
    # causal triangle is read and written, the strip i < j < S of valid rows is zero-filled.  Not on the
    # layer's path (the fused attention never materialises scores): measured for its own roofline row,
    # on as many heads as fit 2 GB.
    S = w.padded_len
    nh = max(1, min(w.heads, int((2 << 30) // (2 * B * S * S))))
    sc = torch.randn(B, nh, S, S, device="cuda:0").half()
    ms = time_launches(torch, lambda: eet.eet_op_softmax_maskfree(sc, stack.lens, 0.125), 4, replays=2)
    tri = sum(L * (L + 1) / 2 for L in stack.lens)
    out.append({"kernel": f"softmax_maskfree_vec: stand-alone mask-free softmax (Algorithm 1), {nh} head(s), not on the layer path",
                "bound": "hbm", "work": nh * (2.0 * 2 * tri + 2.0 * sum(L * S - L * (L + 1) / 2 for L in stack.lens)),
                "ms": ms, "launches": 0})
    # (6b) stand-alone add-bias + GELU over [T, F] rows and add-bias + residual over [T, H] rows (the kernels the paper
    # runs between its library GEMM calls; here they are epilogues, so these launches are not on the layer path):
    # 4F resp. 6H bytes per token (+ the bias row)
    del sc
    del yp
    gi = torch.randn(T, F, device="cuda:0").half()
    go = torch.empty_like(gi)
    ms = time_launches(torch, lambda: eet.eet_op_bias_gelu(gi, stack.weights(0)["b_fc1"], go), max(4, min(reps, 16)), replays=2)
    out.append({"kernel": f"bias_act_vec<false>: stand-alone add-bias + GELU over {T} rows of {F}, not on the layer path",
                "bound": "hbm", "work": 4.0 * T * F + 2.0 * F, "ms": ms, "launches": 0})
    del go, gi
    ro = torch.empty_like(rh)
    ms = time_launches(torch, lambda: eet.eet_op_bias_residual(xp, stack.weights(0)["b_o"], rh, ro), max(4, min(reps, 16)), replays=2)
    out.append({"kernel": f"bias_act_vec<true>: stand-alone add-bias + residual over {T} rows of {H}, not on the layer path",
                "bound": "hbm", "work": 6.0 * T * H + 2.0 * H, "ms": ms, "launches": 0})
    del ro
    # (7) the operators around the stack at GPT-2's vocabulary (50257, padded to 50304 columns): not on the layer pass
    # that the metric counts, measured for their own roofline rows.  Skipped where the table would pass 512 MB.
    V, Vp = 50257, 50304
    if w.decode_steps and 2 * Vp * H <= (512 << 20):
        wte = torch.randn(Vp, H, device="cuda:0").half().mul_(0.02)
        wpe = torch.randn(w.max_seq, H, device="cuda:0").half().mul_(0.01)
        ids = torch.randint(0, V, (B, S), dtype=torch.int32, device="cuda:0")
        emb = torch.empty(B, S, H, device="cuda:0", dtype=torch.float16)
        ms = time_launches(torch, lambda: eet.eet_op_embedding(ids, stack.lens, wte, wpe, emb, vocab=V), 8, replays=2)
        out.append({"kernel": "embed_tokens: token + position embedding of the prompts (pad rows zero-filled), not on the layer path",
                    "bound": "hbm", "work": 6.0 * T * H + 2.0 * (B * S - T) * H + 4.0 * T, "ms": ms, "launches": 0})
        xh = torch.randn(B, H, device="cuda:0").half()
        zb = torch.zeros(Vp, device="cuda:0", dtype=torch.float16)
        lg = torch.empty(B, Vp, device="cuda:0", dtype=torch.float16)
        tables = [wte] + [wte.clone() for _ in range(3)]      # four copies in turn: none is still in a cache when its turn comes
        st7 = {"i": 0}

        def run_head():
            st7["i"] += 1
            eet.eet_op_linear(xh, tables[st7["i"] % 4], zb, lg)
        ms = time_launches(torch, run_head, 8, replays=2)
        out.append({"kernel": f"decode output projection over the vocabulary (weight stream, M = {B} rows, N = {Vp}), not on the layer path",
                    "bound": "hbm", "work": 2.0 * (Vp * H + B * H + Vp + B * Vp), "ms": ms, "launches": 0})
        nxt = torch.empty(B, device="cuda:0", dtype=torch.int32)
        ms = time_launches(torch, lambda: eet.eet_op_argmax(lg, nxt, vocab=V), 16, replays=2)
        out.append({"kernel": f"argmax_rows: greedy choice over {B} rows of {V} logits, not on the layer path",
                    "bound": "hbm", "work": 2.0 * B * V + 4.0 * B, "ms": ms, "launches": 0})
    return out


def roofline_for(stack, torch, eet, reps, full=True):
    """Roofline record of the dominant kernel (largest share of the pass) and of the others.  `achieved` divides the
    algorithmic work of one launch by the launch duration measured live in this run; `traffic` is the profiled HBM bytes
    per launch from the committed counter summary of the workload (null when there is none), with its source."""
    recs = []
    measured, source = profiled_traffic(stack.w.name)
    for c in _kernel_candidates(stack, torch, eet, reps, full):
        if c["bound"] == "hbm":
            ach, peak, unit = c["work"] / (c["ms"] * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = c["work"] / (c["ms"] * 1e-3) / 1e12, MFMA_FP16_PEAK_TFLOPS, "TFLOP/s"
        traffic = next((v for k, v in measured.items() if c["kernel"].startswith(k)), None)
        recs.append({"kernel": c["kernel"], "bound": c["bound"], "achieved": ach, "peak": peak, "unit": unit,
                     "frac": ach / peak, "traffic": traffic, "traffic_source": source if traffic is not None else None,
                     "avg_launch_us": c["ms"] * 1e3,
                     "algorithmic_work_per_launch": c["work"], "share_ms_per_pass": c["ms"] * c["launches"]})
    recs.sort(key=lambda r: -r["share_ms_per_pass"])
    return recs[0], recs[1:]


def hbm_reference(torch):
    """What a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + bytes written per
    second): context for the HBM fractions, which divide by the published 8 TB/s."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(3)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ms = time_region(torch, lambda: dst.copy_(src), 5)
    return {"kind": "device-to-device copy of 1 GiB (read + write bytes)", "GB/s": 2.0 * (1 << 30) / (ms * 1e-3) / 1e9}


def cpu_baseline(w, wl, budget_s=25.0, min_s=10.0):
    """The CPU oracle timed on a bounded sample of the same workload: whole layers (as many as it
    takes to reach about ten seconds, at most the stack), as many whole sequences as fit a flop
    budget, and decode steps until the time budget is used.  The result is scaled to whole-stack
    tokens/s (time per layer multiplied by the number of layers)."""
    import numpy as np

    from oracle import eet_oracle as orc
    flop_budget = 5.0e12                                          # ten to twenty seconds of float64 matrix products per layer on the host cores
    lens_all = wl.lengths(w)
    flops_seq = 24.0 * lens_all.astype(np.float64) * w.hidden * w.hidden
    nseq = 1
    while nseq < w.batch and flops_seq[: nseq + 1].sum() <= flop_budget:
        nseq += 1
    lens = lens_all[:nseq].copy()
    cut = ""
    if flops_seq[0] > flop_budget:        # one prompt alone is beyond the budget: its causal prefix is a smaller prompt of the same kind
        keep = max(64, int(flop_budget / (24.0 * w.hidden * w.hidden)) // 64 * 64)
        cut = f", prompt cut to its first {keep} of {int(lens[0])} tokens"
        lens[0] = keep
    weights = [{k: v.astype(np.float64) for k, v in wl.layer_weights(w, li).items()} for li in range(min(w.layers, 4))]
    x = wl.prompt_embeddings(w)[:nseq]
    dec = [wl.decode_embeddings(w, k)[:nseq] for k in range(w.decode_steps)]
    total, layers_done, steps_done, tokens = 0.0, 0, [], 0
    while layers_done < w.layers and total < min_s:
        oracle = orc.DecoderLayerOracle(weights[layers_done % len(weights)], w.heads, nseq, w.max_seq, w.ln_eps)
        t0 = time.perf_counter()
        oracle.encode(x, lens) if w.encoder else oracle.prefill(x, lens)
        steps = 0
        while steps < w.decode_steps and time.perf_counter() - t0 < budget_s:
            oracle.decode_step(dec[steps])
            steps += 1
        total += time.perf_counter() - t0
        layers_done += 1
        steps_done.append(steps)
        tokens += int(lens.sum()) + nseq * steps
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        nthreads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        nthreads = cores
    per_layer_tokens = tokens / layers_done
    return {"value": per_layer_tokens / (total / layers_done * w.layers), "unit": "tokens/s",
            "cores": min(cores, nthreads), "kind": "oracle",
            "sample": f"float64 oracle, {layers_done} of {w.layers} layer(s) (time per layer scaled by {w.layers}), "
                      f"{nseq} of {w.batch} sequences (lengths {lens.tolist()}{cut}), prefill + {steps_done[0]} of "
                      f"{w.decode_steps} decode steps each; {total:.1f} s of CPU work, {tokens} layer-tokens"}


def workload_text(w, model=False):
    return (f"{w.name}: {w.layers} layer(s), hidden {w.hidden}, heads {w.heads}, ffn {w.ffn}, batch {w.batch}, prompts "
            f"{w.len_lo}-{w.len_hi} padded to {w.padded_len}, {w.decode_steps} decode steps, cache {w.max_seq}" +
            (f"; through the model entry points: token ids in, embedding, final LayerNorm, output projection over "
             f"{ModelStack.VOCAB} tokens and greedy choice per step, fed back on the device" if model else ""))


def measure(stack, a, torch, eet, steps, warmup, full):
    """Whole-pass timing (host clock around `steps` passes, everything resident), phase split (HIP events on the launch
    stream) and per-kernel roofline records of one workload."""
    w = stack.w
    tokens = sum(stack.lens) + w.batch * w.decode_steps       # valid tokens only
    for _ in range(warmup):
        stack.one_pass()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        stack.one_pass()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_prefill = time_region(torch, stack.prefill, 2, stack.stream)
    ms_decode = time_region(torch, stack.decode, 1, stack.stream) if w.decode_steps else 0.0
    rec = {"value": tokens / (dt / steps), "unit": "tokens/s", "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3,
           "config": {"workload": workload_text(w, a.model), "valid_tokens_per_step": tokens, "prefill_tokens": sum(stack.lens),
                      "decode_tokens": w.batch * w.decode_steps, "prefill_ms": ms_prefill, "decode_ms": ms_decode,
                      "prefill_tokens_per_s": sum(stack.lens) / (ms_prefill * 1e-3),
                      "decode_tokens_per_s": (w.batch * w.decode_steps) / (ms_decode * 1e-3) if ms_decode else None}}
    rec["roofline"], rec["roofline_other_kernels"] = roofline_for(stack, torch, eet, a.kernel_reps, full)
    return rec


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (asked for --gpus {a.gpus}); sharding by sequence is a "
              "design note, not code", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2104_12470_amd import eet, workloads as wl
    eet.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    w = wl.WORKLOADS[a.workload]
    if a.model and (w.encoder or not w.decode_steps):
        print("bench.py: --model needs a decoder workload with decode steps", file=sys.stderr)
        sys.exit(2)
    shared = {}                              # device weights by (seed, shape): cfg5a and cfg5b are one layer on two batches

    def build(wk, model=False):
        if wk.encoder:
            return EncoderStack(wk, eet, torch, wl)
        if model:
            return ModelStack(wk, eet, torch, wl, use_graph=not a.no_graph)
        key = (wk.seed, wk.hidden, wk.heads, wk.ffn, wk.layers, wk.sigma_w)
        if key not in shared:
            shared[key] = [{k: torch.from_numpy(v).to("cuda:0") for k, v in wl.layer_weights(wk, li).items()}
                           for li in range(wk.layers)]
        return Stack(wk, eet, torch, wl, use_graph=not a.no_graph, device_weights=shared[key])

    stack = build(w, a.model)
    if a.roofline_only:
        stack.one_pass() if w.decode_steps <= 64 else stack.prefill()   # caches hold real keys/values
        # plain copy kernel of known size under a name nothing else in the run uses: x + 0 over
        # 256 MiB of int32 reads 256 MiB and writes 256 MiB
        src = torch.ones(64 << 20, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.add(src, 0, out=dst)
        torch.cuda.synchronize()
        main_rec, others = roofline_for(stack, torch, eet, a.kernel_reps)
        print(json.dumps({"workload": w.name, "roofline": main_rec, "roofline_other_kernels": others, "copy_bytes": 256 << 20}))
        return

    m = measure(stack, a, torch, eet, a.steps, a.warmup, full=True)
    rec = {
        "metric": ("encoder-layer tokens/s (one pass, no sequence mask) fp16; % of HBM/MFMA roofline" if w.encoder else
                   "decoder-layer tokens/s (prefill+decode) fp16; % of HBM/MFMA roofline"),
        "value": m["value"], "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic", "config": m["config"],
        "roofline": m["roofline"], "roofline_other_kernels": m["roofline_other_kernels"],
    }
    rec["hbm_reference"] = hbm_reference(torch)
    del stack
    torch.cuda.empty_cache()
    # the other workloads, same measurement, two timed passes each
    others = {}
    for name in [n for n in a.also.split(",") if n and n != a.workload]:
        wk = wl.WORKLOADS[name]
        st = build(wk)
        others[name] = measure(st, a, torch, eet, 2, 1, full=False)
        del st
        torch.cuda.empty_cache()
    if others:
        rec["other_workloads"] = others
    shared.clear()
    torch.cuda.empty_cache()
    if not a.no_cpu_baseline and not a.model:      # the timed oracle sample is the layer stack's, not the model's
        rec["cpu_baseline"] = cpu_baseline(w, wl)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
