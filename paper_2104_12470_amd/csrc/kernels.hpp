// Host-side launchers of the gfx950 kernels.  Each launcher validates nothing: the C-ABI
// layer in eet_api.hip checks shapes and pointers before any launch.
#pragma once

#include "common.hpp"

namespace eet {

// ---- row-wise kernels (rowops.hip) ---------------------------------------------------------
// LayerNorm of `rows` rows.  Row r is read from x[in_row_map ? in_row_map[r] : r] and written
// to y[r].  If bump_lens != nullptr, the block of row r < bump_count also does bump_lens[r] += 1
// (advances the per-sequence cache length after all readers of this step were enqueued).
hipError_t launch_layernorm(const half_t* x, const int32_t* in_row_map, const half_t* gamma,
                            const half_t* beta, half_t* y, int64_t rows, int width, float eps,
                            int32_t* bump_lens, int bump_count, hipStream_t s);
hipError_t launch_bias_gelu(const half_t* x, const half_t* bias, half_t* y, int64_t rows, int width,
                            hipStream_t s);
hipError_t launch_bias_residual(const half_t* x, const half_t* bias, const half_t* res, half_t* y,
                                int64_t rows, int width, hipStream_t s);
// left_padded: the valid positions of sequence b are S-len[b] .. S-1 (the layout Algorithm 1 is printed for)
hipError_t launch_softmax_maskfree(half_t* scores, const SeqLens& lens, int batch, int heads, int S,
                                   float scale, hipStream_t s, bool left_padded = false);
// Index set-up of a prefill: device copies of the lengths, prefix sums, packed->padded row map,
// and zero fill of the pad rows of `out` ([batch, S, width]).
hipError_t launch_prefill_setup(const SeqLens& lens, int batch, int S, int width, int32_t* cache_lens,
                                int32_t* cu_seqlens, int32_t* row_map, half_t* out, hipStream_t s,
                                bool left_padded = false);

// cache_lens[b] = lens.len[b] for b < batch (DEVICE array of the layer's workspace)
hipError_t launch_set_cache_lens(const SeqLens& lens, int batch, int32_t* cache_lens, hipStream_t s);

// ---- operands of the launches that follow, pulled towards the memory-side cache -------------
// A latency-bound decode projection leaves CUs idle (64-128 workgroups on 256 CUs).  Extra workgroups of the same
// launch use them to touch one word of every 128-byte line of what the NEXT launches will read (weights; the K/V
// rows of the next attention): those launches then find their operands in the memory-side cache, at about half
// the latency of HBM.  Nothing depends on it: the data is read and dropped.
struct PrefetchArgs {
    const void* lin[2];         // linear ranges ...
    uint32_t lin_lines[2];      // ... in 128-byte lines
    const half_t* k_cache;      // K/V rows [0, lens[b]) of every (sequence, head); nullptr = none
    const half_t* v_cache;
    const int32_t* lens;        // DEVICE
    int kv_batch, kv_heads, kv_d, kv_capacity;
    int blocks;                 // extra workgroups that do nothing else; 0 = no prefetch
};

// ---- dense projections (gemm.hip) ------------------------------------------------------------
enum Epilogue : int { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RES = 2, EPI_QKV = 3 };

struct GemmArgs {
    const half_t* x;        // [M, K] activations, row-major
    const half_t* w;        // [N, K] weights, row-major
    const half_t* bias;     // [N]
    half_t* y;              // output [*, N] (EPI_QKV: the Q rows, [M, hidden])
    int M, N, K;
    // MFMA tile kernels only (launch_gemm refuses them elsewhere; see gemm_takes_row_strides): halfs between consecutive
    // rows of x and of y (0: K and N; multiples of 8, not below K and N; not with EPI_QKV)
    int lda, ldy;
    // EPI_BIAS_RES: residual row of output row m is res[res_row_map ? res_row_map[m] : m]
    const half_t* res;
    const int32_t* res_row_map;
    // output row of m is out_row_map ? out_row_map[m] : m   (scatter back to the padded layout)
    const int32_t* out_row_map;
    // EPI_QKV: columns [0,hidden) -> y, [hidden,2*hidden) -> K cache, [2*hidden,3*hidden) -> V cache.
    // Row m belongs to (b, pos): prefill: (row_map[m] / S, row_map[m] % S); decode: (m, lens[m]).
    half_t* k_cache;
    half_t* v_cache;
    const int32_t* tok_row_map;   // prefill: packed row -> b*S + pos ; nullptr in decode
    const int32_t* lens;          // decode: device cache lengths; prefill with left_pad: device prompt lengths
    int left_pad;                 // prefill: tokens of sequence b sit at rows S-len[b] .. S-1 of its block (position = row - (S-len[b]))
    int S, hidden, heads, d, max_seq;
    // weight-streaming kernel only (M <= 16): LayerNorm of x fused in front (nullptr = x is used as it is),
    // and n_b += 1 for the first bump_count sequences (nullptr = no)
    const half_t* ln_gamma;
    const half_t* ln_beta;
    float ln_eps;
    int32_t* bump_lens;
    int bump_count;
    PrefetchArgs pf;              // gemm_flat only
    // gemm_flat with EPI_BIAS_RES only (x_splits > 1): the activations are the decode attention's output still split
    // over key ranges, and the kernel merges the ranges while it loads them (x is not read).  Row m, head g = column
    // / d, range s: weighted values x_part_acc[((m*heads + g)*x_splits + s)*d ..+d], (maximum, sum) in the exp2
    // domain x_part_ml[((m*heads + g)*x_splits + s)*2 ..+2]; heads and d above give the layout.
    const float* x_part_acc;
    const float* x_part_ml;
    int x_splits;
    // gemm_stream with at most 16 rows only: the statistics of a LayerNorm handed from the projection that writes a row
    // (EPI_BIAS_RES, row_stats_out != nullptr) to the projection that normalises it (ln_gamma != nullptr, row_stats_in !=
    // nullptr), so that no launch stands between the two.  Every workgroup of the producer also writes, per row, the mean
    // and the sum of squared deviations of its own columns of the rounded output: row_stats_out[(group*16 + row)*2 ..+2].
    // The consumer merges the row_stats_groups groups of row_stats_cols columns each into mean and 1/std per row and
    // normalises the activation rows on their way to the matrix instructions; its x is the producer's output as it is.
    float* row_stats_out;
    const float* row_stats_in;
    int row_stats_groups, row_stats_cols;
    // gemm_stream only: 1 = the weights are read with the non-temporal hint (common.hpp: load_once).  Right when nothing
    // could keep them cached until their next use anyway (a decode step that moves more than the memory-side cache holds);
    // wrong for a layer small enough to live in that cache from step to step, which the hint would keep out of it.
    int read_once;
};
// the memory-side cache of the part: what a decode step must exceed, in bytes moved between two uses of an operand, before
// its read-once operands are loaded with the non-temporal hint
constexpr size_t kMemorySideCacheBytes = (size_t)256 << 20;
// For a bias+residual projection that launch_gemm would give to gemm_stream and that then can leave row statistics for
// `consumer` (which gemm_stream must take too): the layout of row_stats_out (workgroups, columns per workgroup); else false.
bool gemm_hands_row_stats(const GemmArgs& producer, const GemmArgs& consumer, Epilogue consumer_epi, int& groups, int& cols);
// true when launch_gemm can serve this problem with row strides (more than 16 rows: an MFMA tile kernel)
bool gemm_takes_row_strides(const GemmArgs& a);
// true when launch_gemm would give this bias+residual projection to the kernel that can merge the key ranges itself
bool gemm_merges_attention_ranges(const GemmArgs& a);

// M > 16: MFMA tile kernel.  M <= 16 (decode): weight-streaming kernel.
hipError_t launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s);

// ---- attention (attention.hip) -------------------------------------------------------------------
// Prefill: q rows of sequence b start at q_row0 + b*q_seq_stride (+ prefix sum of lens if packed).
struct AttnPrefillArgs {
    const half_t* q;        // row r, head g at q[r*hidden + g*d]
    half_t* ctx;            // same addressing as q
    const half_t* k_cache;  // [batch, heads, capacity, d]
    const half_t* v_cache;
    int batch, heads, d, capacity, hidden;
    int packed;             // 1: rows of sequence b start at sum(len[0..b)); 0: at b*S
    int S;                  // padded length (row stride between sequences when not packed)
    int max_len;            // max over lens (sizes the grid)
    int causal;             // 1: query i sees keys 0..i; 0: every valid query sees all L_b keys (encoder)
    int chunk_pairs, chunk_tiles;   // set by the launcher (callers leave 0): the grid order of the prefill kernels
};
hipError_t launch_attention_prefill(const AttnPrefillArgs& a, const SeqLens& lens, hipStream_t s);
// Unfused form (causal, not packed, S a multiple of 8): raw scores q.k into scores[batch, heads, S, S] for the tiles
// Algorithm 1 will look at; and ctx = probs . V from the probabilities Algorithm 1 left there.
hipError_t launch_attention_scores(const AttnPrefillArgs& a, const SeqLens& lens, half_t* scores, hipStream_t s);
hipError_t launch_attention_apply(const AttnPrefillArgs& a, const SeqLens& lens, const half_t* probs, hipStream_t s);

struct AttnDecodeArgs {
    const half_t* q;        // [batch, heads*d]
    half_t* ctx;            // [batch, heads*d]
    const half_t* k_cache;
    const half_t* v_cache;
    const int32_t* lens;    // DEVICE: number of visible keys minus `len_bias`
    int len_bias;           // keys visible = lens[b] + len_bias (1 inside a decode step: the new token)
    int batch, heads, d, capacity;
    int splits;             // key-range splits per (sequence, head)
    float* part_acc;        // [batch*heads*splits, d]   (splits > 1)
    float* part_ml;         // [batch*heads*splits, 2]
    int leave_ranges;       // 1: no merge launch, the projection that follows merges the ranges (GemmArgs::x_splits)
    int read_once;          // 1: K/V rows loaded with the non-temporal hint (see GemmArgs::read_once)
};
int attention_decode_splits(int batch, int heads, int capacity);
size_t attention_decode_scratch_bytes(int batch, int heads, int d, int splits);
hipError_t launch_attention_decode(const AttnDecodeArgs& a, hipStream_t s);

// ---- operators around the stack (model.hip) ------------------------------------------------------
// out[b*S + i] = wte[ids[b*S + i]] + wpe[i - first] for first <= i < first + lens.len[b] (first = 0, or S - lens.len[b]
// when left_padded), zeros for pad rows (positions == nullptr);
// or, with S == 1, out[b] = wte[ids[b]] + wpe[positions[b]] (positions on the DEVICE).  Rows whose id or position
// is outside its table become NaN.  last_row (optional, DEVICE [batch]): row index of each sequence's last valid token.
hipError_t launch_embedding(const int32_t* ids, const SeqLens& lens, const int32_t* positions, int batch, int S, int width,
                            int vocab, int max_pos, const half_t* wte, const half_t* wpe, half_t* out, int32_t* last_row,
                            hipStream_t s, bool left_padded = false);
// out[r] = first maximum of logits[r*ld + 0 .. vocab)   (ld % 8 == 0)
hipError_t launch_argmax(const half_t* logits, int rows, int vocab, int ld, int32_t* out, hipStream_t s);

}  // namespace eet
