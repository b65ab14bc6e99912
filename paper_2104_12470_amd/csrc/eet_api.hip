// C ABI of the library (declared in include/eet.h): argument validation, workspace carve-up,
// launch sequencing.  No device allocation, no synchronisation except eet_cache_lens.
#include "../../include/eet.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "kernels.hpp"

using namespace eet;

static_assert(EET_MAX_BATCH == kMaxBatch, "header and kernels disagree on the batch limit");

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what) {
    return fail(EET_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Rows of the prefill's feed-forward buffer lie F + kFfnRowPad halfs apart when F >= kFfnPadFrom: rows a
// multiple of 32 KB apart slow the second feed-forward projection down (25082 x 12288 x 49152: 0.97-1.09 PFLOP/s with
// rows 96 KB apart, 1.16 with 128 bytes more; no gain at 16384 and below, a small loss at 4096).
// The operator entry points do not know what else runs between two of their calls: an operand of this size or more
// (weights of a projection, the K/V capacity of a decode attention) is taken to come from HBM every time and is read with
// the non-temporal hint; the layer, stack and model entry points decide from what a whole decode step moves.
constexpr size_t kReadOnceOperandBytes = (size_t)64 << 20;
constexpr size_t kFfnRowPad = 64;
constexpr int kFfnPadFrom = 32768;

// Byte offsets of the pieces of a layer's workspace.
struct WorkspaceLayout {
    size_t lens, cu, row_map, buf_a, buf_b, buf_y, buf_f, part, row_stats, total;
    int splits;
};

const char* config_problem(const eet_layer_config* c) {
    if (!c) return "config is null";
    if (c->hidden <= 0 || c->heads <= 0 || c->ffn <= 0) return "hidden, heads and ffn must be positive";
    if (c->hidden % c->heads != 0) return "hidden must be a multiple of heads";
    if (c->max_batch < 1 || c->max_prompt < 1 || c->max_seq < 1) return "capacities must be positive";
    if (!(c->ln_eps > 0.f)) return "ln_eps must be positive";
    return nullptr;
}

const char* shape_problem(const eet_layer_config* c) {
    const int d = c->hidden / c->heads;
    if (d != 64 && d != 128) return "head size must be 64 or 128";
    if (c->ffn % 64 != 0) return "ffn must be a multiple of 64";
    if (c->max_batch > EET_MAX_BATCH) return "max_batch exceeds EET_MAX_BATCH";
    if (c->max_seq < c->max_prompt) return "max_seq must be at least max_prompt";
    if ((int64_t)c->max_batch * c->max_prompt > (int64_t)1 << 30) return "max_batch*max_prompt too large";
    return nullptr;
}

WorkspaceLayout layout_of(const eet_layer_config* c) {
    WorkspaceLayout w{};
    const size_t T = (size_t)c->max_batch * c->max_prompt, H = c->hidden, F = c->ffn;
    size_t off = 0;
    w.lens = off;    off = align_up(off + sizeof(int32_t) * EET_MAX_BATCH, 256);
    w.cu = off;      off = align_up(off + sizeof(int32_t) * (EET_MAX_BATCH + 1), 256);
    w.row_map = off; off = align_up(off + sizeof(int32_t) * T, 256);
    w.buf_a = off;   off = align_up(off + 2 * T * H, 256);
    w.buf_b = off;   off = align_up(off + 2 * T * H, 256);
    w.buf_y = off;   off = align_up(off + 2 * T * H, 256);
    w.buf_f = off;   off = align_up(off + 2 * T * (F + kFfnRowPad), 256);
    w.splits = attention_decode_splits(c->max_batch, c->heads, c->max_seq);
    w.part = off;
    // sized for the split count of any batch <= max_batch (fewer sequences -> more splits)
    size_t part = 0;
    for (int b = 1; b <= c->max_batch; ++b) {
        const size_t p = attention_decode_scratch_bytes(b, c->heads, H / c->heads,
                                                        attention_decode_splits(b, c->heads, c->max_seq));
        part = p > part ? p : part;
    }
    off = align_up(off + part, 256);
    // LayerNorm statistics handed from the output projection of a decode step to the first feed-forward projection:
    // (mean, squared deviations) per row and workgroup of the producer, at most hidden/16 workgroups of 16 rows
    w.row_stats = off;
    off = align_up(off + (H / 16 + 1) * 16 * 2 * sizeof(float), 256);
    w.total = off;
    return w;
}

}  // namespace

struct eet_layer {
    eet_layer_config cfg;
    eet_layer_weights w;
    WorkspaceLayout lay;
    char* ws;
    int d;
    int batch;                         // batch of the last prefill, 0 = none yet
    int stack_layers;                  // layers whose decode steps run between two steps of this one (1: a layer on its own)
    int32_t host_lens[EET_MAX_BATCH];  // host mirror of the device cache lengths (capacity checks only)
};

// error setter for the library's other translation units (same thread-local message as eet_last_error)
int eet_set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" {

const char* eet_last_error(void) { return g_err; }

size_t eet_kv_cache_bytes(const eet_layer_config* cfg) {
    if (config_problem(cfg)) return 0;
    return (size_t)2 * cfg->max_batch * cfg->hidden * cfg->max_seq * sizeof(half_t);
}

size_t eet_workspace_bytes(const eet_layer_config* cfg) {
    if (config_problem(cfg) || shape_problem(cfg)) return 0;
    return layout_of(cfg).total;
}

int eet_layer_create(const eet_layer_config* cfg, const eet_layer_weights* weights, void* workspace,
                     eet_layer_t** out_layer) {
    if (!out_layer) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: out_layer is null");
    *out_layer = nullptr;
    if (const char* p = config_problem(cfg)) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: %s", p);
    if (const char* p = shape_problem(cfg)) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_layer_create: %s", p);
    if (!weights || !workspace) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: weights or workspace is null");
    const void* const* wp = reinterpret_cast<const void* const*>(weights);
    for (size_t i = 0; i < sizeof(eet_layer_weights) / sizeof(void*); ++i) {
        if (!wp[i]) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: weight pointer %zu is null", i);
        if (!aligned16(wp[i])) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: weight pointer %zu is not 16-byte aligned", i);
    }
    if (reinterpret_cast<uintptr_t>(workspace) & 255u)
        return fail(EET_ERR_INVALID_ARG, "eet_layer_create: workspace is not 256-byte aligned");
    eet_layer* L = new (std::nothrow) eet_layer();
    if (!L) return fail(EET_ERR_INVALID_ARG, "eet_layer_create: out of host memory");
    L->cfg = *cfg;
    L->w = *weights;
    L->lay = layout_of(cfg);
    L->ws = static_cast<char*>(workspace);
    L->d = cfg->hidden / cfg->heads;
    L->batch = 0;
    std::memset(L->host_lens, 0, sizeof(L->host_lens));
    *out_layer = L;
    g_err[0] = 0;
    return EET_OK;
}

int eet_layer_destroy(eet_layer_t* layer) {
    delete layer;
    return EET_OK;
}

#define EET_LAUNCH(expr, what)                        \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) return hip_fail(e_, what); \
    } while (0)

// Enqueue the kernels of one layer's prefill (arguments already validated).
// index_setup = false: a layer of a stack whose workspace already holds this prefill's lengths, prefix sums and row map
// and whose output buffer already has its pad rows zeroed (an earlier layer of the same call did both).
static int enqueue_prefill(eet_layer* L, const SeqLens& lens, int batch, int padded_len, int64_t T, int max_len,
                           const void* tokens, void* out, void* kv_cache, hipStream_t s, bool causal = true,
                           bool left_padded = false, bool index_setup = true) {
    const eet_layer_config& c = L->cfg;
    const int H = c.hidden, F = c.ffn;
    int32_t* d_lens = reinterpret_cast<int32_t*>(L->ws + L->lay.lens);
    int32_t* d_cu = reinterpret_cast<int32_t*>(L->ws + L->lay.cu);
    int32_t* d_map = reinterpret_cast<int32_t*>(L->ws + L->lay.row_map);
    half_t* bufA = reinterpret_cast<half_t*>(L->ws + L->lay.buf_a);
    half_t* bufB = reinterpret_cast<half_t*>(L->ws + L->lay.buf_b);
    half_t* bufY = reinterpret_cast<half_t*>(L->ws + L->lay.buf_y);
    half_t* bufF = reinterpret_cast<half_t*>(L->ws + L->lay.buf_f);
    const half_t* x = static_cast<const half_t*>(tokens);
    half_t* kc = static_cast<half_t*>(kv_cache);
    half_t* vc = kc + (size_t)c.max_batch * H * c.max_seq;

    // a1: padding offsets -> integers on the device; pad rows of `out` zeroed
    // (left_padded: the packed->padded row map starts each sequence at row S - L_b; every kernel below works on
    // the packed rows and never sees the difference, except the cache scatter, which needs the position)
    if (index_setup)
        EET_LAUNCH(launch_prefill_setup(lens, batch, padded_len, H, d_lens, d_cu, d_map, static_cast<half_t*>(out), s,
                                        left_padded), "prefill_setup");
    // a2: LN1 over valid rows only (gathered into the packed layout)
    EET_LAUNCH(launch_layernorm(x, d_map, (const half_t*)L->w.ln1_g, (const half_t*)L->w.ln1_b, bufA, T, H, c.ln_eps,
                                nullptr, 0, s), "layernorm 1");
    // a3: QKV projection; K and V rows land directly in their cache slots
    GemmArgs g{};
    g.x = bufA; g.w = (const half_t*)L->w.w_qkv; g.bias = (const half_t*)L->w.b_qkv; g.y = bufB;
    g.M = (int)T; g.N = 3 * H; g.K = H;
    g.k_cache = kc; g.v_cache = vc; g.tok_row_map = d_map; g.lens = left_padded ? d_lens : nullptr;
    g.left_pad = left_padded ? 1 : 0;
    g.S = padded_len; g.hidden = H; g.heads = c.heads; g.d = L->d; g.max_seq = c.max_seq;
    EET_LAUNCH(launch_gemm(g, EPI_QKV, s), "qkv projection");
    // a4: mask-free attention over the cache (causal window, or all valid keys for the encoder)
    AttnPrefillArgs at{};
    at.q = bufB; at.ctx = bufA; at.k_cache = kc; at.v_cache = vc;
    at.batch = batch; at.heads = c.heads; at.d = L->d; at.capacity = c.max_seq; at.hidden = H;
    at.packed = 1; at.S = padded_len; at.max_len = max_len; at.causal = causal ? 1 : 0;
    EET_LAUNCH(launch_attention_prefill(at, lens, s), "prefill attention");
    // a6: output projection + bias + residual (residual gathered from the padded input)
    GemmArgs o{};
    o.x = bufA; o.w = (const half_t*)L->w.w_o; o.bias = (const half_t*)L->w.b_o; o.y = bufY;
    o.M = (int)T; o.N = H; o.K = H; o.res = x; o.res_row_map = d_map;
    EET_LAUNCH(launch_gemm(o, EPI_BIAS_RES, s), "output projection");
    // a7: LN2
    EET_LAUNCH(launch_layernorm(bufY, nullptr, (const half_t*)L->w.ln2_g, (const half_t*)L->w.ln2_b, bufB, T, H,
                                c.ln_eps, nullptr, 0, s), "layernorm 2");
    // a8: FFN1 + bias + GELU
    GemmArgs f1{};
    f1.x = bufB; f1.w = (const half_t*)L->w.w_fc1; f1.bias = (const half_t*)L->w.b_fc1; f1.y = bufF;
    f1.M = (int)T; f1.N = F; f1.K = H;
    // a9: FFN2 + bias + residual, scattered back to the padded layout
    GemmArgs f2{};
    f2.x = bufF; f2.w = (const half_t*)L->w.w_fc2; f2.bias = (const half_t*)L->w.b_fc2; f2.y = static_cast<half_t*>(out);
    f2.M = (int)T; f2.N = H; f2.K = F; f2.res = bufY; f2.res_row_map = nullptr; f2.out_row_map = d_map;
    if (F >= kFfnPadFrom && gemm_takes_row_strides(f1) && gemm_takes_row_strides(f2)) f1.ldy = f2.lda = F + (int)kFfnRowPad;
    EET_LAUNCH(launch_gemm(f1, EPI_BIAS_GELU, s), "ffn 1");
    EET_LAUNCH(launch_gemm(f2, EPI_BIAS_RES, s), "ffn 2");

    return EET_OK;
}

// Shared argument checks of a prefill; fills the by-value length table.
static int check_prefill(const char* who, const eet_layer_config& cfg, const int32_t* q_lens, int32_t batch,
                         int32_t padded_len, const void* tokens, const void* out, const void* kv_cache, SeqLens& lens,
                         int64_t& T, int& max_len) {
    if (!q_lens || !tokens || !out || !kv_cache) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || padded_len < 1) return fail(EET_ERR_INVALID_ARG, "%s: batch and padded_len must be >= 1", who);
    if (batch > cfg.max_batch) return fail(EET_ERR_CAPACITY, "%s: batch %d > max_batch %d", who, batch, cfg.max_batch);
    if (padded_len > cfg.max_prompt)
        return fail(EET_ERR_CAPACITY, "%s: padded_len %d > max_prompt %d", who, padded_len, cfg.max_prompt);
    if (!aligned16(tokens) || !aligned16(out) || !aligned16(kv_cache))
        return fail(EET_ERR_INVALID_ARG, "%s: tokens/out/kv_cache must be 16-byte aligned", who);
    std::memset(&lens, 0, sizeof(lens));
    T = 0;
    max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] < 1 || q_lens[b] > padded_len)
            return fail(EET_ERR_INVALID_ARG, "%s: q_lens[%d] = %d outside [1, %d]", who, b, q_lens[b], padded_len);
        lens.len[b] = q_lens[b];
        T += q_lens[b];
        max_len = q_lens[b] > max_len ? q_lens[b] : max_len;
    }
    return EET_OK;
}

int eet_prefill(eet_layer_t* L, const int32_t* q_lens, int32_t batch, int32_t padded_len, const void* tokens,
                void* out, void* kv_cache, void* hip_stream) {
    if (!L) return fail(EET_ERR_INVALID_ARG, "eet_prefill: null argument");
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill("eet_prefill", L->cfg, q_lens, batch, padded_len, tokens, out, kv_cache, lens, T, max_len))
        return rc;
    const int rc = enqueue_prefill(L, lens, batch, padded_len, T, max_len, tokens, out, kv_cache,
                                   static_cast<hipStream_t>(hip_stream));
    if (rc != EET_OK) return rc;
    L->batch = batch;
    for (int b = 0; b < batch; ++b) L->host_lens[b] = q_lens[b];
    return EET_OK;
}

int eet_prefill_left_padded(eet_layer_t* L, const int32_t* q_lens, int32_t batch, int32_t padded_len, const void* tokens,
                            void* out, void* kv_cache, void* hip_stream) {
    if (!L) return fail(EET_ERR_INVALID_ARG, "eet_prefill_left_padded: null argument");
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill("eet_prefill_left_padded", L->cfg, q_lens, batch, padded_len, tokens, out, kv_cache, lens, T,
                                     max_len))
        return rc;
    const int rc = enqueue_prefill(L, lens, batch, padded_len, T, max_len, tokens, out, kv_cache,
                                   static_cast<hipStream_t>(hip_stream), true, true);
    if (rc != EET_OK) return rc;
    L->batch = batch;
    for (int b = 0; b < batch; ++b) L->host_lens[b] = q_lens[b];
    return EET_OK;
}

int eet_layer_encode(eet_layer_t* L, const int32_t* q_lens, int32_t batch, int32_t padded_len, const void* tokens,
                     void* out, void* kv_scratch, void* hip_stream) {
    if (!L) return fail(EET_ERR_INVALID_ARG, "eet_layer_encode: layer is null");
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill("eet_layer_encode", L->cfg, q_lens, batch, padded_len, tokens, out, kv_scratch, lens, T, max_len))
        return rc;
    // the pass overwrites the device-side lengths: whatever prefill / decode state the layer held is gone
    L->batch = 0;
    return enqueue_prefill(L, lens, batch, padded_len, T, max_len, tokens, out, kv_scratch,
                           static_cast<hipStream_t>(hip_stream), false);
}

// Enqueue the kernels of one layer's decode step (arguments already validated).  `bump`: this
// layer advances the device-side cache lengths (in a stack only the last layer does).
static int enqueue_decode(eet_layer* L, const void* tokens, void* out, void* kv_cache, hipStream_t s, bool bump,
                          const eet_layer* next = nullptr, const void* next_kv = nullptr) {
    const eet_layer_config& c = L->cfg;
    const int B = L->batch, H = c.hidden, F = c.ffn;
    int32_t* d_lens = reinterpret_cast<int32_t*>(L->ws + L->lay.lens);
    half_t* bufA = reinterpret_cast<half_t*>(L->ws + L->lay.buf_a);
    half_t* bufB = reinterpret_cast<half_t*>(L->ws + L->lay.buf_b);
    half_t* bufY = reinterpret_cast<half_t*>(L->ws + L->lay.buf_y);
    half_t* bufF = reinterpret_cast<half_t*>(L->ws + L->lay.buf_f);
    const half_t* x = static_cast<const half_t*>(tokens);
    half_t* kc = static_cast<half_t*>(kv_cache);
    half_t* vc = kc + (size_t)c.max_batch * H * c.max_seq;

    // Small layers are launch-bound in decode: there the two LayerNorms run inside the projections
    // that consume them (each workgroup recomputes the row statistics of the <= 16 token rows).
    // Measured break-even is near 16 MB of FFN-1 weights; larger layers keep the separate row kernel.
    const bool fuse_ln = B <= 16 && (size_t)F * H * sizeof(half_t) <= ((size_t)16 << 20);
    // What a decode step moves between two uses of the same weight or cache row: every layer's weights and visible K/V
    // once.  More than the memory-side cache holds: nothing survives there until the next step, and the read-once operands
    // are loaded with the non-temporal hint (a tenth faster from HBM).  Less (hidden 2048 on its own: 150 MB): the step
    // lives in that cache, which the hint would only disturb (6.68 -> 6.75 ms for 128 steps).
    size_t visible = 0;
    for (int b = 0; b < B; ++b) visible += (size_t)L->host_lens[b] + 1;
    const size_t step_bytes = (size_t)(L->stack_layers > 0 ? L->stack_layers : 1) *
                              (2 * ((size_t)4 * H * H + (size_t)2 * H * F) + (size_t)4 * H * visible);
    // (not for the small layers whose idle workgroups pull the next launches' operands into that cache: PrefetchArgs below;
    // the hint on the consumer's loads undoes that: 24 hidden-1024 layers 320.7 -> 330.4 ms for 512 steps)
    const int once = (step_bytes > kMemorySideCacheBytes && !fuse_ln) ? 1 : 0;
    // The same small layers leave CUs idle in every launch: extra workgroups of the two launches with the fewest
    // workgroups pull operands of later launches towards the memory-side cache (PrefetchArgs).  `next`: the layer
    // whose step follows this one (the next layer of a stack, or this layer's own next step).  Measured on the
    // 24-layer hidden-1024 stack, one call: 346 -> 324 ms for 512 decode steps.  Prefetching during the attention or
    // the QKV projection, other workgroup counts (64, 96, 112, 192, 256) and the first feed-forward matrix instead
    // of the second were all slower: the attention streams from HBM itself, and 128 keeps main plus extra
    // workgroups at one per CU.  Moving any share of the K/V rows (a quarter to all) from FFN-2's extra workgroups to
    // the output projection's was slower too (324 -> 361-367 ms).
    constexpr int kPrefetchBlocks = 128;
    const bool prefetch = fuse_ln;
    auto lines = [](size_t bytes) { return (uint32_t)(bytes / 128); };
    const half_t* qkv_in = x;
    if (!fuse_ln) {
        EET_LAUNCH(launch_layernorm(x, nullptr, (const half_t*)L->w.ln1_g, (const half_t*)L->w.ln1_b, bufA, B, H,
                                    c.ln_eps, nullptr, 0, s), "layernorm 1");
        qkv_in = bufA;
    }
    GemmArgs g{};
    g.x = qkv_in; g.w = (const half_t*)L->w.w_qkv; g.bias = (const half_t*)L->w.b_qkv; g.y = bufB;
    g.M = B; g.N = 3 * H; g.K = H;
    g.k_cache = kc; g.v_cache = vc; g.tok_row_map = nullptr; g.lens = d_lens;   // new token -> slot n_b
    g.S = 1; g.hidden = H; g.heads = c.heads; g.d = L->d; g.max_seq = c.max_seq; g.read_once = once;
    if (fuse_ln) { g.ln_gamma = (const half_t*)L->w.ln1_g; g.ln_beta = (const half_t*)L->w.ln1_b; g.ln_eps = c.ln_eps; }
    EET_LAUNCH(launch_gemm(g, EPI_QKV, s), "qkv projection");
    AttnDecodeArgs at{};
    at.q = bufB; at.ctx = bufA; at.k_cache = kc; at.v_cache = vc; at.lens = d_lens; at.len_bias = 1;
    at.batch = B; at.heads = c.heads; at.d = L->d; at.capacity = c.max_seq; at.read_once = once;
    at.splits = attention_decode_splits(B, c.heads, c.max_seq);
    at.part_acc = reinterpret_cast<float*>(L->ws + L->lay.part);
    at.part_ml = at.part_acc + (size_t)B * c.heads * at.splits * L->d;
    // output projection + bias + residual; its first workgroup also advances n_b: every reader of
    // n_b in this step (cache append, attention) is already ordered before it on the stream
    GemmArgs o{};
    o.x = bufA; o.w = (const half_t*)L->w.w_o; o.bias = (const half_t*)L->w.b_o; o.y = bufY;
    o.M = B; o.N = H; o.K = H; o.res = x; o.read_once = once;
    o.heads = c.heads; o.d = L->d;
    // With the key range split (few (sequence, head) pairs) the ranges need merging.  Where the output projection goes to
    // the small-layer kernel, that kernel merges them while it loads its activations, and the merge launch (4 us, the
    // floor of a dependent launch) is gone; otherwise attn_decode_combine runs.
    if (at.splits > 1 && gemm_merges_attention_ranges(o)) {
        at.leave_ranges = 1;
        o.x_part_acc = at.part_acc; o.x_part_ml = at.part_ml; o.x_splits = at.splits;
    }
    EET_LAUNCH(launch_attention_decode(at, s), "decode attention");
    const bool bump_in_gemm = B <= 16;
    if (bump && bump_in_gemm) { o.bump_lens = d_lens; o.bump_count = B; }
    if (prefetch) {                                       // during the output projection (64 workgroups): the second feed-forward matrix
        o.pf.lin[0] = L->w.w_fc2; o.pf.lin_lines[0] = lines((size_t)H * F * 2);
        o.pf.blocks = kPrefetchBlocks;
    }
    // Large layers: the second LayerNorm has no launch of its own either when both projections around it go to the
    // weight-streaming kernel: the output projection leaves the statistics of the rows it writes, the first feed-forward
    // projection normalises them on the way in (one launch and its gap less per step: 9 us of hidden 12288's 830, 5 of
    // hidden 4096's 107).
    GemmArgs f1{};
    f1.w = (const half_t*)L->w.w_fc1; f1.bias = (const half_t*)L->w.b_fc1; f1.y = bufF;
    f1.M = B; f1.N = F; f1.K = H; f1.read_once = once;
    bool hand_stats = false;
    if (!fuse_ln && bump_in_gemm) {
        GemmArgs probe = f1;
        probe.x = bufY; probe.ln_gamma = (const half_t*)L->w.ln2_g; probe.ln_beta = (const half_t*)L->w.ln2_b; probe.ln_eps = c.ln_eps;
        int groups = 0, cols = 0;
        if (gemm_hands_row_stats(o, probe, EPI_BIAS_GELU, groups, cols)) {
            hand_stats = true;
            o.row_stats_out = reinterpret_cast<float*>(L->ws + L->lay.row_stats);
            f1 = probe;
            f1.row_stats_in = o.row_stats_out; f1.row_stats_groups = groups; f1.row_stats_cols = cols;
        }
    }
    EET_LAUNCH(launch_gemm(o, EPI_BIAS_RES, s), "output projection");
    if (!hand_stats) {
        const half_t* fc1_in = bufY;
        if (!fuse_ln || !bump_in_gemm) {
            EET_LAUNCH(launch_layernorm(bufY, nullptr, (const half_t*)L->w.ln2_g, (const half_t*)L->w.ln2_b, bufB, B, H,
                                        c.ln_eps, (bump && !bump_in_gemm) ? d_lens : nullptr, B, s), "layernorm 2");
            fc1_in = bufB;
        }
        f1.x = fc1_in;
        if (fc1_in == bufY) { f1.ln_gamma = (const half_t*)L->w.ln2_g; f1.ln_beta = (const half_t*)L->w.ln2_b; f1.ln_eps = c.ln_eps; }
    }
    EET_LAUNCH(launch_gemm(f1, EPI_BIAS_GELU, s), "ffn 1");
    GemmArgs f2{};
    f2.x = bufF; f2.w = (const half_t*)L->w.w_fc2; f2.bias = (const half_t*)L->w.b_fc2; f2.y = static_cast<half_t*>(out);
    f2.M = B; f2.N = H; f2.K = F; f2.res = bufY; f2.read_once = once;
    if (prefetch && next != nullptr) {                    // during FFN-2 (128 workgroups): the QKV matrix and the K/V rows of the step that follows
        f2.pf.lin[0] = next->w.w_qkv; f2.pf.lin_lines[0] = lines((size_t)3 * H * H * 2);
        f2.pf.k_cache = static_cast<const half_t*>(next_kv);
        f2.pf.v_cache = f2.pf.k_cache + (size_t)c.max_batch * H * c.max_seq;
        f2.pf.lens = d_lens;
        f2.pf.kv_batch = B; f2.pf.kv_heads = c.heads; f2.pf.kv_d = L->d; f2.pf.kv_capacity = c.max_seq;
        f2.pf.blocks = kPrefetchBlocks;
    }
    EET_LAUNCH(launch_gemm(f2, EPI_BIAS_RES, s), "ffn 2");
    return EET_OK;
}

int eet_decode_step(eet_layer_t* L, const void* tokens, void* out, void* kv_cache, void* hip_stream) {
    if (!L || !tokens || !out || !kv_cache) return fail(EET_ERR_INVALID_ARG, "eet_decode_step: null argument");
    if (L->batch == 0) return fail(EET_ERR_STATE, "eet_decode_step: no prefill has been run on this layer");
    if (!aligned16(tokens) || !aligned16(out) || !aligned16(kv_cache))
        return fail(EET_ERR_INVALID_ARG, "eet_decode_step: tokens/out/kv_cache must be 16-byte aligned");
    const eet_layer_config& c = L->cfg;
    const int B = L->batch;
    for (int b = 0; b < B; ++b)
        if (L->host_lens[b] + 1 > c.max_seq)
            return fail(EET_ERR_CAPACITY, "eet_decode_step: sequence %d is at the cache capacity %d", b, c.max_seq);
    const int rc = enqueue_decode(L, tokens, out, kv_cache, static_cast<hipStream_t>(hip_stream), true, L, kv_cache);
    if (rc != EET_OK) return rc;
    for (int b = 0; b < B; ++b) L->host_lens[b] += 1;
    return EET_OK;
}

static int check_restore(const char* who, const eet_layer_config& c, const int32_t* lens_host, int32_t batch, SeqLens& lens) {
    if (!lens_host) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1) return fail(EET_ERR_INVALID_ARG, "%s: batch must be >= 1", who);
    if (batch > c.max_batch) return fail(EET_ERR_CAPACITY, "%s: batch %d > max_batch %d", who, batch, c.max_batch);
    std::memset(&lens, 0, sizeof(lens));
    for (int b = 0; b < batch; ++b) {
        if (lens_host[b] < 1 || lens_host[b] > c.max_seq)
            return fail(EET_ERR_INVALID_ARG, "%s: cache_lens[%d] = %d outside [1, %d]", who, b, lens_host[b], c.max_seq);
        lens.len[b] = lens_host[b];
    }
    return EET_OK;
}

int eet_restore(eet_layer_t* L, const int32_t* cache_lens, int32_t batch, void* hip_stream) {
    if (!L) return fail(EET_ERR_INVALID_ARG, "eet_restore: null argument");
    SeqLens lens;
    if (const int rc = check_restore("eet_restore", L->cfg, cache_lens, batch, lens)) return rc;
    EET_LAUNCH(launch_set_cache_lens(lens, batch, reinterpret_cast<int32_t*>(L->ws + L->lay.lens), static_cast<hipStream_t>(hip_stream)),
               "set cache lengths");
    L->batch = batch;
    for (int b = 0; b < batch; ++b) L->host_lens[b] = cache_lens[b];
    return EET_OK;
}

int eet_cache_lens(eet_layer_t* L, int32_t* out_host, void* hip_stream) {
    if (!L || !out_host) return fail(EET_ERR_INVALID_ARG, "eet_cache_lens: null argument");
    if (L->batch == 0) return fail(EET_ERR_STATE, "eet_cache_lens: no prefill has been run on this layer");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    EET_LAUNCH(hipMemcpyAsync(out_host, L->ws + L->lay.lens, sizeof(int32_t) * L->batch, hipMemcpyDeviceToHost, s),
               "copy of cache lengths");
    EET_LAUNCH(hipStreamSynchronize(s), "stream synchronise");
    return EET_OK;
}

// ------------------------------------------------------------------------------------------------
// a stack of layers
// ------------------------------------------------------------------------------------------------
struct eet_stack {
    eet_layer_config cfg;
    int n_layers;
    eet_layer** layers;                // every layer borrows the same scratch: they run one after another
    char* ws;
    size_t act[2];                     // byte offsets of the two inter-layer activation buffers
    size_t layer_cache_bytes;
    int batch;
    int32_t host_lens[EET_MAX_BATCH];
    int use_graph;
    hipGraphExec_t exec;               // captured decode step, valid for (g_tokens, g_out, g_kv, g_batch)
    const void* g_tokens;
    void* g_out;
    void* g_kv;
    int g_batch;
};

static size_t stack_act_bytes(const eet_layer_config* c) {
    return align_up((size_t)2 * c->max_batch * c->max_prompt * c->hidden, 256);
}

size_t eet_stack_kv_cache_bytes(const eet_layer_config* cfg, int32_t n_layers) {
    if (n_layers < 1) return 0;
    return eet_kv_cache_bytes(cfg) * (size_t)n_layers;
}

size_t eet_stack_workspace_bytes(const eet_layer_config* cfg, int32_t n_layers) {
    if (n_layers < 1 || config_problem(cfg) || shape_problem(cfg)) return 0;
    return layout_of(cfg).total + 2 * stack_act_bytes(cfg);
}

int eet_stack_destroy(eet_stack_t* st) {
    if (!st) return EET_OK;
    if (st->exec) (void)hipGraphExecDestroy(st->exec);
    if (st->layers) {
        for (int l = 0; l < st->n_layers; ++l) delete st->layers[l];
        delete[] st->layers;
    }
    delete st;
    return EET_OK;
}

int eet_stack_create(const eet_layer_config* cfg, int32_t n_layers, const eet_layer_weights* weights, void* workspace,
                     int32_t use_graph, eet_stack_t** out_stack) {
    if (!out_stack) return fail(EET_ERR_INVALID_ARG, "eet_stack_create: out_stack is null");
    *out_stack = nullptr;
    if (n_layers < 1) return fail(EET_ERR_INVALID_ARG, "eet_stack_create: n_layers must be >= 1");
    if (!weights) return fail(EET_ERR_INVALID_ARG, "eet_stack_create: weights is null");
    eet_stack* st = new (std::nothrow) eet_stack();
    if (!st) return fail(EET_ERR_INVALID_ARG, "eet_stack_create: out of host memory");
    st->layers = new (std::nothrow) eet_layer*[n_layers]();
    st->n_layers = n_layers;
    if (!st->layers) {
        eet_stack_destroy(st);
        return fail(EET_ERR_INVALID_ARG, "eet_stack_create: out of host memory");
    }
    for (int l = 0; l < n_layers; ++l) {
        const int rc = eet_layer_create(cfg, &weights[l], workspace, &st->layers[l]);
        if (rc != EET_OK) {
            eet_stack_destroy(st);
            return rc;
        }
        st->layers[l]->stack_layers = n_layers;
    }
    st->cfg = *cfg;
    st->ws = static_cast<char*>(workspace);
    st->act[0] = layout_of(cfg).total;
    st->act[1] = st->act[0] + stack_act_bytes(cfg);
    st->layer_cache_bytes = eet_kv_cache_bytes(cfg);
    st->batch = 0;
    st->use_graph = use_graph != 0;
    st->exec = nullptr;
    *out_stack = st;
    return EET_OK;
}

// The layers of a stack share one workspace, so the index set-up of layer 0 (lengths, prefix sums, row map) serves them
// all; what is left per layer is zeroing the pad rows of its output buffer.  Layers 0 and 1 do that for the two
// activation buffers the stack alternates between (nothing writes a pad row afterwards: the last projection of a layer
// scatters valid rows only), the last layer for the caller's buffer; the layers in between skip the launch.
static bool stack_layer_needs_setup(int l, int n_layers) { return l < 2 || l == n_layers - 1; }

static int stack_prefill(const char* who, bool left_padded, eet_stack_t* st, const int32_t* q_lens, int32_t batch,
                         int32_t padded_len, const void* tokens, void* out, void* kv_cache, void* hip_stream) {
    if (!st) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill(who, st->cfg, q_lens, batch, padded_len, tokens, out, kv_cache, lens, T, max_len))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const void* in = tokens;
    for (int l = 0; l < st->n_layers; ++l) {
        void* o = (l == st->n_layers - 1) ? out : static_cast<void*>(st->ws + st->act[l & 1]);
        char* kv = static_cast<char*>(kv_cache) + (size_t)l * st->layer_cache_bytes;
        const int rc = enqueue_prefill(st->layers[l], lens, batch, padded_len, T, max_len, in, o, kv, s, true, left_padded,
                                       stack_layer_needs_setup(l, st->n_layers));
        if (rc != EET_OK) return rc;
        st->layers[l]->batch = batch;
        in = o;
    }
    st->batch = batch;
    for (int b = 0; b < batch; ++b) st->host_lens[b] = q_lens[b];
    return EET_OK;
}

int eet_stack_prefill(eet_stack_t* st, const int32_t* q_lens, int32_t batch, int32_t padded_len, const void* tokens,
                      void* out, void* kv_cache, void* hip_stream) {
    return stack_prefill("eet_stack_prefill", false, st, q_lens, batch, padded_len, tokens, out, kv_cache, hip_stream);
}

int eet_stack_prefill_left_padded(eet_stack_t* st, const int32_t* q_lens, int32_t batch, int32_t padded_len,
                                  const void* tokens, void* out, void* kv_cache, void* hip_stream) {
    return stack_prefill("eet_stack_prefill_left_padded", true, st, q_lens, batch, padded_len, tokens, out, kv_cache, hip_stream);
}

int eet_stack_encode(eet_stack_t* st, const int32_t* q_lens, int32_t batch, int32_t padded_len, const void* tokens,
                     void* out, void* kv_scratch, void* hip_stream) {
    if (!st) return fail(EET_ERR_INVALID_ARG, "eet_stack_encode: null argument");
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill("eet_stack_encode", st->cfg, q_lens, batch, padded_len, tokens, out, kv_scratch, lens, T, max_len))
        return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    st->batch = 0;                                   // the pass overwrites the device-side lengths: no decode state afterwards
    const void* in = tokens;
    for (int l = 0; l < st->n_layers; ++l) {
        void* o = (l == st->n_layers - 1) ? out : static_cast<void*>(st->ws + st->act[l & 1]);
        st->layers[l]->batch = 0;
        // every layer's keys and values of this pass go to the same scratch: the layers run one after another
        const int rc = enqueue_prefill(st->layers[l], lens, batch, padded_len, T, max_len, in, o, kv_scratch, s, false, false,
                                       stack_layer_needs_setup(l, st->n_layers));
        if (rc != EET_OK) return rc;
        in = o;
    }
    return EET_OK;
}

static int stack_enqueue_decode(eet_stack* st, const void* tokens, void* out, void* kv_cache, hipStream_t s) {
    const void* in = tokens;
    for (int l = 0; l < st->n_layers; ++l) {
        const bool last = l == st->n_layers - 1;
        void* o = last ? out : static_cast<void*>(st->ws + st->act[l & 1]);
        char* kv = static_cast<char*>(kv_cache) + (size_t)l * st->layer_cache_bytes;
        const int ln = last ? 0 : l + 1;                                    // the step that follows this layer's
        const int rc = enqueue_decode(st->layers[l], in, o, kv, s, last,    // lengths shared: advanced once, at the end
                                      st->layers[ln], static_cast<char*>(kv_cache) + (size_t)ln * st->layer_cache_bytes);
        if (rc != EET_OK) return rc;
        in = o;
    }
    return EET_OK;
}

int eet_stack_decode_step(eet_stack_t* st, const void* tokens, void* out, void* kv_cache, void* hip_stream) {
    if (!st || !tokens || !out || !kv_cache) return fail(EET_ERR_INVALID_ARG, "eet_stack_decode_step: null argument");
    if (st->batch == 0) return fail(EET_ERR_STATE, "eet_stack_decode_step: no prefill has been run on this stack");
    if (!aligned16(tokens) || !aligned16(out) || !aligned16(kv_cache))
        return fail(EET_ERR_INVALID_ARG, "eet_stack_decode_step: tokens/out/kv_cache must be 16-byte aligned");
    const int B = st->batch;
    for (int b = 0; b < B; ++b)
        if (st->host_lens[b] + 1 > st->cfg.max_seq)
            return fail(EET_ERR_CAPACITY, "eet_stack_decode_step: sequence %d is at the cache capacity %d", b, st->cfg.max_seq);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // A step has no host-varying argument (the cache lengths live on the device), so its launches
    // can be recorded once and replayed.  Not on the null stream (it cannot be captured) and not
    // while the caller is capturing this stream itself (then the launches join the caller's graph).
    bool graph = st->use_graph && s != nullptr;
    if (graph) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) graph = false;
    }
    if (!graph) {
        if (const int rc = stack_enqueue_decode(st, tokens, out, kv_cache, s)) return rc;
    } else {
        if (st->exec && (st->g_tokens != tokens || st->g_out != out || st->g_kv != kv_cache || st->g_batch != B)) {
            (void)hipGraphExecDestroy(st->exec);
            st->exec = nullptr;
        }
        if (!st->exec) {
            hipGraph_t g = nullptr;
            EET_LAUNCH(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal), "begin capture");
            const int rc = stack_enqueue_decode(st, tokens, out, kv_cache, s);
            const hipError_t e = hipStreamEndCapture(s, &g);
            if (rc != EET_OK) {
                if (g) (void)hipGraphDestroy(g);
                return rc;
            }
            if (e != hipSuccess) return hip_fail(e, "end capture");
            const hipError_t ei = hipGraphInstantiate(&st->exec, g, nullptr, nullptr, 0);
            (void)hipGraphDestroy(g);
            if (ei != hipSuccess) {
                st->exec = nullptr;
                return hip_fail(ei, "graph instantiate");
            }
            st->g_tokens = tokens; st->g_out = out; st->g_kv = kv_cache; st->g_batch = B;
        }
        EET_LAUNCH(hipGraphLaunch(st->exec, s), "graph launch");
    }
    for (int b = 0; b < B; ++b) st->host_lens[b] += 1;
    return EET_OK;
}

int eet_stack_restore(eet_stack_t* st, const int32_t* cache_lens, int32_t batch, void* hip_stream) {
    if (!st) return fail(EET_ERR_INVALID_ARG, "eet_stack_restore: null argument");
    SeqLens lens;
    if (const int rc = check_restore("eet_stack_restore", st->cfg, cache_lens, batch, lens)) return rc;
    eet_layer* L0 = st->layers[0];                       // the layers share one set of device-side lengths
    EET_LAUNCH(launch_set_cache_lens(lens, batch, reinterpret_cast<int32_t*>(L0->ws + L0->lay.lens), static_cast<hipStream_t>(hip_stream)),
               "set cache lengths");
    for (int l = 0; l < st->n_layers; ++l) st->layers[l]->batch = batch;
    st->batch = batch;
    for (int b = 0; b < batch; ++b) st->host_lens[b] = cache_lens[b];
    return EET_OK;
}

int eet_stack_cache_lens(eet_stack_t* st, int32_t* out_host, void* hip_stream) {
    if (!st || !out_host) return fail(EET_ERR_INVALID_ARG, "eet_stack_cache_lens: null argument");
    if (st->batch == 0) return fail(EET_ERR_STATE, "eet_stack_cache_lens: no prefill has been run on this stack");
    return eet_cache_lens(st->layers[0], out_host, hip_stream);
}

// ------------------------------------------------------------------------------------------------
// the model around a stack
// ------------------------------------------------------------------------------------------------
struct eet_model {
    eet_stack* st;
    eet_model_config mc;
    eet_model_weights w;
    char* ws;
    size_t zero_bias, last_row, x_dec, y_dec, ln_out;   // byte offsets into ws
    const void* hidden_in;                               // what the latest call left behind (see eet_model_hidden_states)
    const void* hidden_out;
};

struct ModelLayout {
    size_t zero_bias, last_row, x_dec, y_dec, ln_out, total;
};

static ModelLayout model_layout(const eet_layer_config* c, const eet_model_config* m) {
    ModelLayout l{};
    const size_t row = align_up((size_t)2 * c->max_batch * c->hidden, 256);
    size_t off = 0;
    l.zero_bias = off; off = align_up(off + (size_t)2 * m->vocab_padded, 256);
    l.last_row = off;  off = align_up(off + sizeof(int32_t) * EET_MAX_BATCH, 256);
    l.x_dec = off;     off += row;
    l.y_dec = off;     off += row;
    l.ln_out = off;    off += row;
    l.total = off;
    return l;
}

static const char* model_config_problem(const eet_model_config* m) {
    if (!m) return "model config is null";
    if (m->vocab < 1 || m->vocab_padded < m->vocab || m->max_pos < 1) return "vocab, vocab_padded >= vocab and max_pos must be positive";
    return nullptr;
}

size_t eet_model_workspace_bytes(const eet_layer_config* cfg, const eet_model_config* mcfg) {
    if (config_problem(cfg) || shape_problem(cfg) || model_config_problem(mcfg) || mcfg->vocab_padded % 64 != 0) return 0;
    return model_layout(cfg, mcfg).total;
}

int eet_model_destroy(eet_model_t* m) {
    delete m;
    return EET_OK;
}

int eet_model_create(eet_stack_t* stack, const eet_layer_config* cfg, const eet_model_config* mcfg,
                     const eet_model_weights* weights, void* workspace, eet_model_t** out_model) {
    if (!out_model) return fail(EET_ERR_INVALID_ARG, "eet_model_create: out_model is null");
    *out_model = nullptr;
    if (!stack || !cfg || !weights || !workspace) return fail(EET_ERR_INVALID_ARG, "eet_model_create: null argument");
    if (const char* p = model_config_problem(mcfg)) return fail(EET_ERR_INVALID_ARG, "eet_model_create: %s", p);
    if (std::memcmp(cfg, &stack->cfg, sizeof(*cfg)) != 0)
        return fail(EET_ERR_INVALID_ARG, "eet_model_create: cfg is not the configuration the stack was created with");
    if (mcfg->vocab_padded % 64 != 0)
        return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_model_create: vocab_padded must be a multiple of 64");
    if (mcfg->max_pos < cfg->max_seq)
        return fail(EET_ERR_INVALID_ARG, "eet_model_create: max_pos %d < max_seq %d of the stack", mcfg->max_pos, cfg->max_seq);
    if (!weights->wte || !weights->wpe || !weights->lnf_g || !weights->lnf_b)
        return fail(EET_ERR_INVALID_ARG, "eet_model_create: a weight pointer is null");
    if (!aligned16(weights->wte) || !aligned16(weights->wpe) || !aligned16(weights->lnf_g) || !aligned16(weights->lnf_b) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return fail(EET_ERR_INVALID_ARG, "eet_model_create: weights must be 16-byte and the workspace 256-byte aligned");
    eet_model* m = new (std::nothrow) eet_model();
    if (!m) return fail(EET_ERR_INVALID_ARG, "eet_model_create: out of host memory");
    const ModelLayout l = model_layout(cfg, mcfg);
    m->st = stack; m->mc = *mcfg; m->w = *weights; m->ws = static_cast<char*>(workspace);
    m->zero_bias = l.zero_bias; m->last_row = l.last_row; m->x_dec = l.x_dec; m->y_dec = l.y_dec; m->ln_out = l.ln_out;
    m->hidden_in = m->hidden_out = nullptr;
    const hipError_t e = hipMemset(m->ws + m->zero_bias, 0, (size_t)2 * mcfg->vocab_padded);
    if (e != hipSuccess) {
        delete m;
        return hip_fail(e, "eet_model_create: clearing the zero bias");
    }
    *out_model = m;
    return EET_OK;
}

// final LayerNorm of `batch` rows of `hidden` (gathered through row_map when given), output projection, greedy choice
static int model_head(eet_model* m, const void* hidden, const int32_t* row_map, int batch, void* logits, int32_t* next_ids,
                      hipStream_t s) {
    const eet_layer_config& c = m->st->cfg;
    half_t* ln = reinterpret_cast<half_t*>(m->ws + m->ln_out);
    EET_LAUNCH(launch_layernorm((const half_t*)hidden, row_map, (const half_t*)m->w.lnf_g, (const half_t*)m->w.lnf_b, ln,
                                batch, c.hidden, c.ln_eps, nullptr, 0, s), "final layernorm");
    GemmArgs g{};
    g.x = ln; g.w = (const half_t*)m->w.wte; g.bias = reinterpret_cast<const half_t*>(m->ws + m->zero_bias);
    g.y = (half_t*)logits; g.M = batch; g.N = m->mc.vocab_padded; g.K = c.hidden;
    EET_LAUNCH(launch_gemm(g, EPI_BIAS, s), "output projection");
    if (next_ids) EET_LAUNCH(launch_argmax((const half_t*)logits, batch, m->mc.vocab, m->mc.vocab_padded, next_ids, s), "greedy choice");
    return EET_OK;
}

static int model_prefill(const char* who, bool left_padded, eet_model_t* m, const int32_t* q_lens, int32_t batch,
                         int32_t padded_len, const int32_t* ids, void* logits, int32_t* next_ids, void* kv_cache,
                         void* hip_stream) {
    if (!m || !ids || !logits) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (!aligned16(logits)) return fail(EET_ERR_INVALID_ARG, "%s: logits must be 16-byte aligned", who);
    eet_stack* st = m->st;
    void* x0 = st->ws + st->act[1];                              // embedding -> one activation cache ...
    void* xn = st->ws + st->act[(st->n_layers - 1) & 1];         // ... final output -> where the last layer's turn falls
    SeqLens lens;
    int64_t T;
    int max_len;
    if (const int rc = check_prefill(who, st->cfg, q_lens, batch, padded_len, x0, xn, kv_cache, lens, T, max_len)) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int32_t* last_row = reinterpret_cast<int32_t*>(m->ws + m->last_row);
    EET_LAUNCH(launch_embedding(ids, lens, nullptr, batch, padded_len, st->cfg.hidden, m->mc.vocab, m->mc.max_pos,
                                (const half_t*)m->w.wte, (const half_t*)m->w.wpe, (half_t*)x0, last_row, s, left_padded), "embedding");
    if (const int rc = stack_prefill(who, left_padded, st, q_lens, batch, padded_len, x0, xn, kv_cache, hip_stream)) return rc;
    m->hidden_in = x0 == xn ? nullptr : x0;      // an even number of layers ends in the buffer the embedding was in
    m->hidden_out = xn;
    return model_head(m, xn, last_row, batch, logits, next_ids, s);
}

int eet_model_prefill(eet_model_t* m, const int32_t* q_lens, int32_t batch, int32_t padded_len, const int32_t* ids,
                      void* logits, int32_t* next_ids, void* kv_cache, void* hip_stream) {
    return model_prefill("eet_model_prefill", false, m, q_lens, batch, padded_len, ids, logits, next_ids, kv_cache, hip_stream);
}

int eet_model_prefill_left_padded(eet_model_t* m, const int32_t* q_lens, int32_t batch, int32_t padded_len,
                                  const int32_t* ids, void* logits, int32_t* next_ids, void* kv_cache, void* hip_stream) {
    return model_prefill("eet_model_prefill_left_padded", true, m, q_lens, batch, padded_len, ids, logits, next_ids, kv_cache,
                         hip_stream);
}

int eet_model_decode_step(eet_model_t* m, const int32_t* ids, void* logits, int32_t* next_ids, void* kv_cache,
                          void* hip_stream) {
    if (!m || !ids || !logits || !kv_cache) return fail(EET_ERR_INVALID_ARG, "eet_model_decode_step: null argument");
    if (!aligned16(logits)) return fail(EET_ERR_INVALID_ARG, "eet_model_decode_step: logits must be 16-byte aligned");
    eet_stack* st = m->st;
    if (st->batch == 0) return fail(EET_ERR_STATE, "eet_model_decode_step: no prefill has been run on this model");
    const int B = st->batch;
    for (int b = 0; b < B; ++b)      // before anything is enqueued (the stack call repeats the check, but after the embedding)
        if (st->host_lens[b] + 1 > st->cfg.max_seq)
            return fail(EET_ERR_CAPACITY, "eet_model_decode_step: sequence %d is at the cache capacity %d", b, st->cfg.max_seq);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    void* x = m->ws + m->x_dec;
    void* y = m->ws + m->y_dec;
    const int32_t* d_lens = reinterpret_cast<const int32_t*>(st->layers[0]->ws + st->layers[0]->lay.lens);
    SeqLens none;
    std::memset(&none, 0, sizeof(none));
    EET_LAUNCH(launch_embedding(ids, none, d_lens, B, 1, st->cfg.hidden, m->mc.vocab, m->mc.max_pos, (const half_t*)m->w.wte,
                                (const half_t*)m->w.wpe, (half_t*)x, nullptr, s), "embedding");
    if (const int rc = eet_stack_decode_step(st, x, y, kv_cache, hip_stream)) return rc;
    m->hidden_in = x;
    m->hidden_out = y;
    return model_head(m, y, nullptr, B, logits, next_ids, s);
}

int eet_model_hidden_states(eet_model_t* m, const void** hidden_in, const void** hidden_out) {
    if (!m) return fail(EET_ERR_INVALID_ARG, "eet_model_hidden_states: null argument");
    if (!m->hidden_out) return fail(EET_ERR_STATE, "eet_model_hidden_states: no call has been run on this model");
    if (hidden_in) *hidden_in = m->hidden_in;
    if (hidden_out) *hidden_out = m->hidden_out;
    return EET_OK;
}

// ------------------------------------------------------------------------------------------------
// operator-level entry points
// ------------------------------------------------------------------------------------------------
int eet_op_layernorm(const void* x, const void* gamma, const void* beta, void* y, int64_t rows, int32_t width,
                     float eps, void* hip_stream) {
    if (!x || !gamma || !beta || !y) return fail(EET_ERR_INVALID_ARG, "eet_op_layernorm: null argument");
    if (rows < 0 || width < 1 || !(eps > 0.f)) return fail(EET_ERR_INVALID_ARG, "eet_op_layernorm: bad size or eps");
    if (rows > 0x7fffffff) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_layernorm: more than 2^31-1 rows");
    EET_LAUNCH(launch_layernorm((const half_t*)x, nullptr, (const half_t*)gamma, (const half_t*)beta, (half_t*)y, rows,
                                width, eps, nullptr, 0, (hipStream_t)hip_stream), "layernorm");
    return EET_OK;
}

static int op_softmax_maskfree(const char* who, bool left_padded, void* scores, const int32_t* q_lens, int32_t batch, int32_t heads,
                               int32_t padded_len, float scale, void* hip_stream) {
    if (!scores || !q_lens) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || heads < 1 || padded_len < 1) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (batch > EET_MAX_BATCH) return fail(EET_ERR_CAPACITY, "%s: batch > EET_MAX_BATCH", who);
    if ((int64_t)batch * heads > 65535) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: batch*heads > 65535", who);
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] < 1 || q_lens[b] > padded_len)
            return fail(EET_ERR_INVALID_ARG, "%s: q_lens[%d] = %d outside [1, %d]", who, b, q_lens[b], padded_len);
        lens.len[b] = q_lens[b];
    }
    EET_LAUNCH(launch_softmax_maskfree((half_t*)scores, lens, batch, heads, padded_len, scale, (hipStream_t)hip_stream,
                                       left_padded), "softmax");
    return EET_OK;
}

int eet_op_softmax_maskfree(void* scores, const int32_t* q_lens, int32_t batch, int32_t heads, int32_t padded_len,
                            float scale, void* hip_stream) {
    return op_softmax_maskfree("eet_op_softmax_maskfree", false, scores, q_lens, batch, heads, padded_len, scale, hip_stream);
}

int eet_op_softmax_maskfree_left_padded(void* scores, const int32_t* q_lens, int32_t batch, int32_t heads,
                                        int32_t padded_len, float scale, void* hip_stream) {
    return op_softmax_maskfree("eet_op_softmax_maskfree_left_padded", true, scores, q_lens, batch, heads, padded_len, scale,
                               hip_stream);
}

int eet_op_bias_gelu(const void* x, const void* bias, void* y, int64_t rows, int32_t width, void* hip_stream) {
    if (!x || !bias || !y) return fail(EET_ERR_INVALID_ARG, "eet_op_bias_gelu: null argument");
    if (rows < 0 || width < 1) return fail(EET_ERR_INVALID_ARG, "eet_op_bias_gelu: bad size");
    EET_LAUNCH(launch_bias_gelu((const half_t*)x, (const half_t*)bias, (half_t*)y, rows, width, (hipStream_t)hip_stream),
               "bias_gelu");
    return EET_OK;
}

int eet_op_bias_residual(const void* x, const void* bias, const void* residual, void* y, int64_t rows, int32_t width,
                         void* hip_stream) {
    if (!x || !bias || !residual || !y) return fail(EET_ERR_INVALID_ARG, "eet_op_bias_residual: null argument");
    if (rows < 0 || width < 1) return fail(EET_ERR_INVALID_ARG, "eet_op_bias_residual: bad size");
    EET_LAUNCH(launch_bias_residual((const half_t*)x, (const half_t*)bias, (const half_t*)residual, (half_t*)y, rows,
                                    width, (hipStream_t)hip_stream), "bias_residual");
    return EET_OK;
}

int eet_op_linear(const void* x, const void* w, const void* bias, const void* residual, void* y, int64_t rows,
                  int32_t in, int32_t out, int32_t act, void* hip_stream) {
    if (!x || !w || !bias || !y) return fail(EET_ERR_INVALID_ARG, "eet_op_linear: null argument");
    if (rows < 0 || in < 1 || out < 1 || (act != 0 && act != 1)) return fail(EET_ERR_INVALID_ARG, "eet_op_linear: bad size or act");
    if (in % 64 != 0 || out % 64 != 0) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_linear: in and out must be multiples of 64");
    if (rows > 0x7fffffff) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_linear: more than 2^31-1 rows");
    if (act == 1 && residual) return fail(EET_ERR_INVALID_ARG, "eet_op_linear: gelu and residual together are not a layer step");
    if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(y) || !aligned16(residual))
        return fail(EET_ERR_INVALID_ARG, "eet_op_linear: pointers must be 16-byte aligned");
    GemmArgs g{};
    g.x = (const half_t*)x; g.w = (const half_t*)w; g.bias = (const half_t*)bias; g.y = (half_t*)y;
    g.M = (int)rows; g.N = out; g.K = in; g.res = (const half_t*)residual;
    g.read_once = (size_t)out * in * sizeof(half_t) >= kReadOnceOperandBytes;
    EET_LAUNCH(launch_gemm(g, residual ? EPI_BIAS_RES : (act ? EPI_BIAS_GELU : EPI_BIAS), (hipStream_t)hip_stream), "linear");
    return EET_OK;
}

int eet_op_linear_strided(const void* x, int64_t ldx, const void* w, const void* bias, const void* residual, void* y, int64_t ldy,
                          int64_t rows, int32_t in, int32_t out, int32_t act, void* hip_stream) {
    if (!x || !w || !bias || !y) return fail(EET_ERR_INVALID_ARG, "eet_op_linear_strided: null argument");
    if (rows < 0 || in < 1 || out < 1 || (act != 0 && act != 1)) return fail(EET_ERR_INVALID_ARG, "eet_op_linear_strided: bad size or act");
    if (in % 64 != 0 || out % 64 != 0) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_linear_strided: in and out must be multiples of 64");
    if (rows > 0x7fffffff) return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_linear_strided: more than 2^31-1 rows");
    if (ldx < in || ldy < out || ldx % 8 != 0 || ldy % 8 != 0 || ldx > 0x7fffffff || ldy > 0x7fffffff)
        return fail(EET_ERR_INVALID_ARG, "eet_op_linear_strided: row strides must be multiples of 8, at least in / out");
    if (act == 1 && residual) return fail(EET_ERR_INVALID_ARG, "eet_op_linear_strided: gelu and residual together are not a layer step");
    if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(y) || !aligned16(residual))
        return fail(EET_ERR_INVALID_ARG, "eet_op_linear_strided: pointers must be 16-byte aligned");
    GemmArgs g{};
    g.x = (const half_t*)x; g.w = (const half_t*)w; g.bias = (const half_t*)bias; g.y = (half_t*)y;
    g.M = (int)rows; g.N = out; g.K = in; g.res = (const half_t*)residual;
    if ((ldx != in || ldy != out) && rows > 0 && !gemm_takes_row_strides(g))
        return fail(EET_ERR_UNSUPPORTED_SHAPE, "eet_op_linear_strided: %lld rows go to the weight-streaming path, which takes dense rows only",
                    (long long)rows);
    g.lda = (int)ldx; g.ldy = (int)ldy;
    g.read_once = (size_t)out * in * sizeof(half_t) >= kReadOnceOperandBytes;
    EET_LAUNCH(launch_gemm(g, residual ? EPI_BIAS_RES : (act ? EPI_BIAS_GELU : EPI_BIAS), (hipStream_t)hip_stream), "linear");
    return EET_OK;
}

static int op_attention_prompt(const char* who, bool causal, const void* q, const void* k_cache, const void* v_cache, void* ctx,
                               const int32_t* q_lens, int32_t batch, int32_t padded_len, int32_t heads, int32_t d,
                               int32_t capacity, void* hip_stream) {
    if (!q || !k_cache || !v_cache || !ctx || !q_lens) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || padded_len < 1 || heads < 1 || capacity < padded_len) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (d != 64 && d != 128) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: head size must be 64 or 128", who);
    if (batch > EET_MAX_BATCH) return fail(EET_ERR_CAPACITY, "%s: batch > EET_MAX_BATCH", who);
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(ctx))
        return fail(EET_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] < 1 || q_lens[b] > padded_len)
            return fail(EET_ERR_INVALID_ARG, "%s: q_lens[%d] = %d outside [1, %d]", who, b, q_lens[b], padded_len);
        lens.len[b] = q_lens[b];
        max_len = q_lens[b] > max_len ? q_lens[b] : max_len;
    }
    AttnPrefillArgs a{};
    a.q = (const half_t*)q; a.ctx = (half_t*)ctx; a.k_cache = (const half_t*)k_cache; a.v_cache = (const half_t*)v_cache;
    a.batch = batch; a.heads = heads; a.d = d; a.capacity = capacity; a.hidden = heads * d;
    a.packed = 0; a.S = padded_len; a.max_len = max_len; a.causal = causal ? 1 : 0;
    EET_LAUNCH(launch_attention_prefill(a, lens, (hipStream_t)hip_stream), "prompt attention");
    return EET_OK;
}

int eet_op_attention_prefill(const void* q, const void* k_cache, const void* v_cache, void* ctx, const int32_t* q_lens,
                             int32_t batch, int32_t padded_len, int32_t heads, int32_t d, int32_t capacity,
                             void* hip_stream) {
    return op_attention_prompt("eet_op_attention_prefill", true, q, k_cache, v_cache, ctx, q_lens, batch, padded_len, heads, d,
                               capacity, hip_stream);
}

int eet_op_attention_encoder(const void* q, const void* k_cache, const void* v_cache, void* ctx, const int32_t* q_lens,
                             int32_t batch, int32_t padded_len, int32_t heads, int32_t d, int32_t capacity,
                             void* hip_stream) {
    return op_attention_prompt("eet_op_attention_encoder", false, q, k_cache, v_cache, ctx, q_lens, batch, padded_len, heads, d,
                               capacity, hip_stream);
}

int eet_op_attention_unfused(const void* q, const void* k_cache, const void* v_cache, void* ctx, const int32_t* q_lens,
                             int32_t batch, int32_t padded_len, int32_t heads, int32_t d, int32_t capacity,
                             eet_bufmgr_t* buffers, int32_t module, void* hip_stream) {
    const char* who = "eet_op_attention_unfused";
    if (!q || !k_cache || !v_cache || !ctx || !q_lens || !buffers) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || padded_len < 1 || heads < 1 || capacity < padded_len) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (d != 64 && d != 128) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: head size must be 64 or 128", who);
    if (padded_len % 8 != 0) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: padded_len must be a multiple of 8", who);
    if (batch > EET_MAX_BATCH) return fail(EET_ERR_CAPACITY, "%s: batch > EET_MAX_BATCH", who);
    if ((int64_t)batch * heads > 65535) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: batch*heads > 65535", who);
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(ctx))
        return fail(EET_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] < 1 || q_lens[b] > padded_len)
            return fail(EET_ERR_INVALID_ARG, "%s: q_lens[%d] = %d outside [1, %d]", who, b, q_lens[b], padded_len);
        lens.len[b] = q_lens[b];
        max_len = q_lens[b] > max_len ? q_lens[b] : max_len;
    }
    void* scores = nullptr;
    const size_t bytes = (size_t)batch * heads * padded_len * padded_len * sizeof(half_t);
    const int rc = eet_bufmgr_request(buffers, bytes, module, &scores);     // the S x S buffer of Section 3.2
    if (rc != EET_OK) return rc;
    AttnPrefillArgs a{};
    a.q = (const half_t*)q; a.ctx = (half_t*)ctx; a.k_cache = (const half_t*)k_cache; a.v_cache = (const half_t*)v_cache;
    a.batch = batch; a.heads = heads; a.d = d; a.capacity = capacity; a.hidden = heads * d;
    a.packed = 0; a.S = padded_len; a.max_len = max_len; a.causal = 1;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_attention_scores(a, lens, (half_t*)scores, s);
    if (e == hipSuccess) e = launch_softmax_maskfree((half_t*)scores, lens, batch, heads, padded_len, 1.0f / std::sqrt((float)d), s);
    if (e == hipSuccess) e = launch_attention_apply(a, lens, (const half_t*)scores, s);
    eet_bufmgr_release(buffers, scores);        // idle for the host; on the stream its next user runs after these kernels
    if (e != hipSuccess) return hip_fail(e, who);
    return EET_OK;
}

static int op_embedding(const char* who, bool left_padded, const int32_t* ids, const int32_t* q_lens, int32_t batch,
                        int32_t padded_len, int32_t hidden, int32_t vocab, int32_t max_pos, const void* wte, const void* wpe,
                        void* out, void* hip_stream) {
    if (!ids || !q_lens || !wte || !wpe || !out) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || padded_len < 1 || hidden < 1 || vocab < 1 || max_pos < 1) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (hidden % 8 != 0) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: hidden must be a multiple of 8", who);
    if (batch > EET_MAX_BATCH) return fail(EET_ERR_CAPACITY, "%s: batch > EET_MAX_BATCH", who);
    if ((int64_t)batch * padded_len > 0x7fffffff) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: more than 2^31-1 rows", who);
    if (!aligned16(wte) || !aligned16(wpe) || !aligned16(out)) return fail(EET_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
    SeqLens lens;
    std::memset(&lens, 0, sizeof(lens));
    for (int b = 0; b < batch; ++b) {
        if (q_lens[b] < 1 || q_lens[b] > padded_len)
            return fail(EET_ERR_INVALID_ARG, "%s: q_lens[%d] = %d outside [1, %d]", who, b, q_lens[b], padded_len);
        lens.len[b] = q_lens[b];
    }
    EET_LAUNCH(launch_embedding(ids, lens, nullptr, batch, padded_len, hidden, vocab, max_pos, (const half_t*)wte,
                                (const half_t*)wpe, (half_t*)out, nullptr, (hipStream_t)hip_stream, left_padded), "embedding");
    return EET_OK;
}

int eet_op_embedding(const int32_t* ids, const int32_t* q_lens, int32_t batch, int32_t padded_len, int32_t hidden,
                     int32_t vocab, int32_t max_pos, const void* wte, const void* wpe, void* out, void* hip_stream) {
    return op_embedding("eet_op_embedding", false, ids, q_lens, batch, padded_len, hidden, vocab, max_pos, wte, wpe, out, hip_stream);
}

int eet_op_embedding_left_padded(const int32_t* ids, const int32_t* q_lens, int32_t batch, int32_t padded_len, int32_t hidden,
                                 int32_t vocab, int32_t max_pos, const void* wte, const void* wpe, void* out, void* hip_stream) {
    return op_embedding("eet_op_embedding_left_padded", true, ids, q_lens, batch, padded_len, hidden, vocab, max_pos, wte, wpe, out,
                        hip_stream);
}

int eet_op_embedding_decode(const int32_t* ids, const int32_t* positions, int32_t batch, int32_t hidden, int32_t vocab,
                            int32_t max_pos, const void* wte, const void* wpe, void* out, void* hip_stream) {
    const char* who = "eet_op_embedding_decode";
    if (!ids || !positions || !wte || !wpe || !out) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || hidden < 1 || vocab < 1 || max_pos < 1) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (hidden % 8 != 0) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: hidden must be a multiple of 8", who);
    if (!aligned16(wte) || !aligned16(wpe) || !aligned16(out)) return fail(EET_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
    SeqLens none;
    std::memset(&none, 0, sizeof(none));
    EET_LAUNCH(launch_embedding(ids, none, positions, batch, 1, hidden, vocab, max_pos, (const half_t*)wte, (const half_t*)wpe,
                                (half_t*)out, nullptr, (hipStream_t)hip_stream), "embedding");
    return EET_OK;
}

int eet_op_argmax(const void* logits, int32_t rows, int32_t vocab, int32_t row_stride, int32_t* out, void* hip_stream) {
    if (!logits || !out) return fail(EET_ERR_INVALID_ARG, "eet_op_argmax: null argument");
    if (rows < 0 || vocab < 1 || row_stride < vocab) return fail(EET_ERR_INVALID_ARG, "eet_op_argmax: bad size");
    if (row_stride % 8 != 0 || !aligned16(logits))
        return fail(EET_ERR_INVALID_ARG, "eet_op_argmax: row_stride must be a multiple of 8 and logits 16-byte aligned");
    EET_LAUNCH(launch_argmax((const half_t*)logits, rows, vocab, row_stride, out, (hipStream_t)hip_stream), "greedy choice");
    return EET_OK;
}

// Shared argument checks of the two decode-attention operators.
static int check_attention_decode(const char* who, const void* q, const void* k_cache, const void* v_cache, const void* ctx,
                                  const int32_t* n_keys, int32_t batch, int32_t heads, int32_t d, int32_t capacity) {
    if (!q || !k_cache || !v_cache || !ctx || !n_keys) return fail(EET_ERR_INVALID_ARG, "%s: null argument", who);
    if (batch < 1 || heads < 1 || capacity < 1) return fail(EET_ERR_INVALID_ARG, "%s: bad size", who);
    if (d != 64 && d != 128) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: head size must be 64 or 128", who);
    if (batch > 65535 || heads > 65535) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: batch or heads > 65535", who);
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(ctx))
        return fail(EET_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", who);
    return EET_OK;
}

size_t eet_op_attention_decode_scratch_bytes(int32_t batch, int32_t heads, int32_t d, int32_t capacity) {
    if (batch < 1 || heads < 1 || d < 1 || capacity < 1) return 0;
    const size_t n = attention_decode_scratch_bytes(batch, heads, d, attention_decode_splits(batch, heads, capacity));
    return n ? n : 256;
}

int eet_op_attention_decode(const void* q, const void* k_cache, const void* v_cache, void* ctx, const int32_t* n_keys,
                            int32_t batch, int32_t heads, int32_t d, int32_t capacity, void* scratch, void* hip_stream) {
    const char* who = "eet_op_attention_decode";
    if (const int rc = check_attention_decode(who, q, k_cache, v_cache, ctx, n_keys, batch, heads, d, capacity)) return rc;
    if (!scratch || !aligned16(scratch)) return fail(EET_ERR_INVALID_ARG, "%s: scratch is null or not 16-byte aligned", who);
    AttnDecodeArgs a{};
    a.q = (const half_t*)q; a.ctx = (half_t*)ctx; a.k_cache = (const half_t*)k_cache; a.v_cache = (const half_t*)v_cache;
    a.lens = n_keys; a.len_bias = 0; a.batch = batch; a.heads = heads; a.d = d; a.capacity = capacity;
    a.read_once = (size_t)4 * batch * heads * d * capacity >= kReadOnceOperandBytes;
    a.splits = attention_decode_splits(batch, heads, capacity);
    a.part_acc = (float*)scratch;
    a.part_ml = a.part_acc + (size_t)batch * heads * a.splits * d;
    EET_LAUNCH(launch_attention_decode(a, (hipStream_t)hip_stream), "decode attention");
    return EET_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// decode attention for callers that cannot allocate
// ------------------------------------------------------------------------------------------------
// The partial results of a split key range live in a device array that is part of the library's code object instead
// of caller memory: every GPU the library runs on holds its own copy, at its own address, until the process ends.
// `scratch` below is only the host-side name of that array: its device address is looked up once per device
// (hipGetSymbolAddress, with that device current) and kept; host code passes the looked-up pointer, never the name.
constexpr size_t kStaticScratchBytes = EET_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Device address of `scratch` on the current device; looked up on the first call per device.
int static_scratch(const char* who, void** out) {
    int dev = -1;
    const hipError_t eg = hipGetDevice(&dev);
    if (eg != hipSuccess) return hip_fail(eg, who);
    if (dev < 0 || dev >= kMaxDevices) return fail(EET_ERR_UNSUPPORTED_SHAPE, "%s: device index %d beyond %d", who, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "address of the library's scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return EET_OK;
}
}  // namespace

extern "C" int eet_op_attention_decode_static(const void* q, const void* k_cache, const void* v_cache, void* ctx,
                                              const int32_t* n_keys, int32_t batch, int32_t heads, int32_t d,
                                              int32_t capacity, void* hip_stream) {
    const char* who = "eet_op_attention_decode_static";
    if (const int rc = check_attention_decode(who, q, k_cache, v_cache, ctx, n_keys, batch, heads, d, capacity)) return rc;
    const int splits = attention_decode_splits(batch, heads, capacity);
    const size_t need = attention_decode_scratch_bytes(batch, heads, d, splits);
    if (need > kStaticScratchBytes)
        return fail(EET_ERR_CAPACITY, "%s: %zu bytes of partial results exceed the library's %zu-byte scratch array "
                    "(use eet_op_attention_decode with a scratch buffer of your own)", who, need, kStaticScratchBytes);
    void* ptr = nullptr;
    if (const int rc = static_scratch(who, &ptr)) return rc;
    AttnDecodeArgs a{};
    a.q = (const half_t*)q; a.ctx = (half_t*)ctx; a.k_cache = (const half_t*)k_cache; a.v_cache = (const half_t*)v_cache;
    a.lens = n_keys; a.len_bias = 0; a.batch = batch; a.heads = heads; a.d = d; a.capacity = capacity;
    a.read_once = (size_t)4 * batch * heads * d * capacity >= kReadOnceOperandBytes;
    a.splits = splits;
    // every slot the merge reads is written by the attention launch in front of it: nothing has to start at zero
    a.part_acc = static_cast<float*>(ptr);
    a.part_ml = a.part_acc + (size_t)batch * heads * splits * d;
    EET_LAUNCH(launch_attention_decode(a, (hipStream_t)hip_stream), "decode attention");
    return EET_OK;
}
