// Operators around the stack of layers (the model-level interface named in the paper's Conclusion; the embedding
// operator and the final output of Section 3.1's activation-cache list): token + position embedding, and the
// greedy choice over a row of logits.  The final LayerNorm and the output projection reuse the row kernel and the
// dense projections.  Both kernels are HBM-bound: 6 * width bytes per embedded token, 2 * vocab bytes per row of logits.
#include <climits>

#include "kernels.hpp"

namespace eet {

// One workgroup per padded row.  Prompt form (positions == nullptr): with first = 0 (right-padded) or S - len[b]
// (left-padded, the layout Algorithm 1 is printed for), row r = b*S + i holds token i - first of sequence b when
// first <= i < first + len[b] (position i - first), otherwise it is a pad row and is written as zeros; its id is never read.  Decode form:
// S == 1, row b holds the new token of sequence b at position positions[b] (the device-side cache length).
// An id outside [0, vocab) or a position outside [0, max_pos) indexes nothing: the row becomes NaN, which every later
// step propagates to the logits.  last_row[b] (optional) receives the row index of the last valid token.
__global__ __launch_bounds__(128) void embed_tokens(const int32_t* __restrict__ ids, SeqLens lens,
                                                    const int32_t* __restrict__ positions, int S, int width, int vocab,
                                                    int max_pos, const half_t* __restrict__ wte,
                                                    const half_t* __restrict__ wpe, half_t* __restrict__ out,
                                                    int32_t* __restrict__ last_row, int left) {
    const int r = blockIdx.x;
    const int b = r / S, i = r % S;
    const int nvec = width >> 3;
    half8v* o = reinterpret_cast<half8v*>(out + (size_t)r * width);
    const int first = (positions == nullptr && left) ? S - lens.len[b] : 0;
    int pos = i - first;
    if (positions != nullptr) {
        pos = positions[b];
    } else if (pos < 0 || pos >= lens.len[b]) {
        half8v z;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = (half_t)0.f;
        for (int c = threadIdx.x; c < nvec; c += 128) o[c] = z;
        return;
    }
    if (last_row != nullptr && threadIdx.x == 0 && (positions != nullptr || pos == lens.len[b] - 1)) last_row[b] = r;
    const int id = ids[r];
    if (id < 0 || id >= vocab || pos < 0 || pos >= max_pos) {
        half8v n;
#pragma unroll
        for (int e = 0; e < 8; ++e) n[e] = (half_t)__builtin_nanf("");
        for (int c = threadIdx.x; c < nvec; c += 128) o[c] = n;
        return;
    }
    const half8v* t = reinterpret_cast<const half8v*>(wte + (size_t)id * width);
    const half8v* p = reinterpret_cast<const half8v*>(wpe + (size_t)pos * width);
    for (int c = threadIdx.x; c < nvec; c += 128) {
        const half8v a = t[c], q = p[c];
        half8v v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (half_t)((float)a[e] + (float)q[e]);     // exact in fp32, rounded once
        o[c] = v;
    }
}

hipError_t launch_embedding(const int32_t* ids, const SeqLens& lens, const int32_t* positions, int batch, int S, int width,
                            int vocab, int max_pos, const half_t* wte, const half_t* wpe, half_t* out, int32_t* last_row,
                            hipStream_t s, bool left_padded) {
    hipLaunchKernelGGL(embed_tokens, dim3(batch * S), dim3(128), 0, s, ids, lens, positions, S, width, vocab, max_pos, wte,
                       wpe, out, last_row, left_padded ? 1 : 0);
    return hipGetLastError();
}

// Greedy choice: out[r] = index of the first maximum of logits[r*ld + 0 .. vocab).  One workgroup of 16 waves per row
// (a decode step has few rows, so a row's 100 KB must come through as many lanes as one workgroup can hold); a thread
// walks its 8-wide chunks in increasing order, so `>` keeps the first of equal values; pairs are merged by
// (larger value, then smaller index).  NaN compares false and never wins; a row with nothing above -inf gives 0.
constexpr int kArgmaxThreads = 1024;
__global__ __launch_bounds__(kArgmaxThreads) void argmax_rows(const half_t* __restrict__ logits, int vocab, int ld,
                                                   int32_t* __restrict__ out) {
    constexpr int NW = kArgmaxThreads / kWave;
    __shared__ float sv[NW];
    __shared__ int si[NW];
    const half_t* row = logits + (size_t)blockIdx.x * ld;
    const int tid = threadIdx.x;
    float best = -__builtin_inff();
    int bi = INT_MAX;
    const int full = vocab >> 3;                                   // whole 8-wide chunks (rows start 16-byte aligned: ld % 8 == 0)
    for (int c = tid; c < full; c += kArgmaxThreads) {
        const half8v v = reinterpret_cast<const half8v*>(row)[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float f = (float)v[e];
            if (f > best) { best = f; bi = c * 8 + e; }
        }
    }
    for (int j = full * 8 + tid; j < vocab; j += kArgmaxThreads) {             // tail: at most 7 columns, one per thread
        const float f = (float)row[j];
        if (f > best) { best = f; bi = j; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o, kWave);
        const int oi = __shfl_xor(bi, o, kWave);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
    }
    if ((tid & 63) == 0) { sv[tid >> 6] = best; si[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < NW; ++w)
            if (sv[w] > best || (sv[w] == best && si[w] < bi)) { best = sv[w]; bi = si[w]; }
        out[blockIdx.x] = bi == INT_MAX ? 0 : bi;
    }
}

hipError_t launch_argmax(const half_t* logits, int rows, int vocab, int ld, int32_t* out, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(argmax_rows, dim3(rows), dim3(kArgmaxThreads), 0, s, logits, vocab, ld, out);
    return hipGetLastError();
}

}  // namespace eet
