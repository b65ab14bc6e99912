// Row-wise kernels: LayerNorm, add-bias+GELU, add-bias+residual, the mask-free softmax of
// Algorithm 1 as a stand-alone operator, and the index set-up of a prefill.
//
// The paper extends these kernels past 1024-wide rows by folding a virtual thread block into
// several real ones (Section 2.2).  On CDNA the same goal is met by folding in time: a fixed
// 256-thread workgroup (or one 64-lane wave for softmax rows) walks the row in 16-byte vectors,
// keeps the row in registers between the reduction and the write when it fits, and re-reads it
// (from L2) when it does not.  Any width works; widths that are a multiple of 8 take the
// vector path.  All of them are HBM-bound: bytes per row = 2 * width * sizeof(fp16).
#include "kernels.hpp"

namespace eet {

// ============================================================================================
// LayerNorm
// ============================================================================================
// NV > 0: each thread caches NV vectors of 8 halfs (width <= NV*2048, width % 8 == 0).
template <int NV>
__global__ __launch_bounds__(256) void layernorm_cached(const half_t* __restrict__ x,
                                                        const int32_t* __restrict__ in_row_map,
                                                        const half_t* __restrict__ gamma,
                                                        const half_t* __restrict__ beta,
                                                        half_t* __restrict__ y, int width, float eps,
                                                        int32_t* bump_lens, int bump_count) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const int64_t src = in_row_map ? (int64_t)in_row_map[row] : row;
    const half8v* xr = reinterpret_cast<const half8v*>(x + src * width);
    const int nvec = width >> 3;
    const int tid = threadIdx.x;

    half8v v[NV];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = tid + i * 256;
        if (idx < nvec) {
            v[i] = xr[idx];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += (float)v[i][e];
        }
    }
    const float mean = block_sum<4>(sum, red) / (float)width;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = tid + i * 256;
        if (idx < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = (float)v[i][e] - mean;
                sq += dlt * dlt;
            }
        }
    }
    const float var = block_sum<4>(sq, red) / (float)width;
    const float rstd = rsqrtf(var + eps);

    const half8v* g8 = reinterpret_cast<const half8v*>(gamma);
    const half8v* b8 = reinterpret_cast<const half8v*>(beta);
    half8v* yr = reinterpret_cast<half8v*>(y + row * width);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = tid + i * 256;
        if (idx < nvec) {
            const half8v g = g8[idx], b = b8[idx];
            half8v o;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                o[e] = (half_t)(((float)v[i][e] - mean) * rstd * (float)g[e] + (float)b[e]);
            yr[idx] = o;
        }
    }
    if (bump_lens != nullptr && tid == 0 && row < bump_count) bump_lens[row] += 1;
}

// Many narrow rows (width <= 2048, width % 8 == 0): one wave per row, four rows per workgroup.  The row sits in NV
// 16-byte vectors per lane, both reductions are lane exchanges, and there is no barrier and no LDS, so a prompt's few
// thousand rows are all in flight at once instead of queueing behind 256-thread workgroups that each wait twice.
template <int NV>
__global__ __launch_bounds__(256) void layernorm_wave(const half_t* __restrict__ x, const int32_t* __restrict__ in_row_map,
                                                      const half_t* __restrict__ gamma, const half_t* __restrict__ beta,
                                                      half_t* __restrict__ y, int rows, int width, float eps,
                                                      int32_t* bump_lens, int bump_count) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;                                  // whole waves leave; nothing below synchronises
    const int64_t src = in_row_map ? (int64_t)in_row_map[row] : (int64_t)row;
    const half8v* xr = reinterpret_cast<const half8v*>(x + src * width);
    const int nvec = width >> 3;
    half8v v[NV];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            v[i] = xr[idx];
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += (float)v[i][e];
        }
    }
    const float mean = wave_sum(sum) / (float)width;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (lane + i * 64 < nvec) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float dlt = (float)v[i][e] - mean;
                sq += dlt * dlt;
            }
        }
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)width + eps);
    const half8v* g8 = reinterpret_cast<const half8v*>(gamma);
    const half8v* b8 = reinterpret_cast<const half8v*>(beta);
    half8v* yr = reinterpret_cast<half8v*>(y + (int64_t)row * width);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + i * 64;
        if (idx < nvec) {
            const half8v g = g8[idx], b = b8[idx];
            half8v o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (half_t)(((float)v[i][e] - mean) * rstd * (float)g[e] + (float)b[e]);
            yr[idx] = o;
        }
    }
    if (bump_lens != nullptr && lane == 0 && row < bump_count) bump_lens[row] += 1;
}

// Any width, any alignment: three scalar passes over the row (re-read through L2).
__global__ __launch_bounds__(256) void layernorm_generic(const half_t* __restrict__ x,
                                                         const int32_t* __restrict__ in_row_map,
                                                         const half_t* __restrict__ gamma,
                                                         const half_t* __restrict__ beta,
                                                         half_t* __restrict__ y, int width, float eps,
                                                         int32_t* bump_lens, int bump_count) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const int64_t src = in_row_map ? (int64_t)in_row_map[row] : row;
    const half_t* xr = x + src * width;
    const int tid = threadIdx.x;
    float sum = 0.f;
    for (int c = tid; c < width; c += 256) sum += (float)xr[c];
    const float mean = block_sum<4>(sum, red) / (float)width;
    float sq = 0.f;
    for (int c = tid; c < width; c += 256) {
        const float dlt = (float)xr[c] - mean;
        sq += dlt * dlt;
    }
    const float var = block_sum<4>(sq, red) / (float)width;
    const float rstd = rsqrtf(var + eps);
    half_t* yr = y + row * width;
    for (int c = tid; c < width; c += 256)
        yr[c] = (half_t)(((float)xr[c] - mean) * rstd * (float)gamma[c] + (float)beta[c]);
    if (bump_lens != nullptr && tid == 0 && row < bump_count) bump_lens[row] += 1;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hipError_t launch_layernorm(const half_t* x, const int32_t* in_row_map, const half_t* gamma,
                            const half_t* beta, half_t* y, int64_t rows, int width, float eps,
                            int32_t* bump_lens, int bump_count, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid((unsigned)rows), block(256);
    const bool vec = (width % 8 == 0) && aligned16(x) && aligned16(y) && aligned16(gamma) && aligned16(beta);
#define EET_LN(NV) hipLaunchKernelGGL(layernorm_cached<NV>, grid, block, 0, s, x, in_row_map, gamma, beta, y, width, eps, bump_lens, bump_count)
#define EET_LNW(NV) hipLaunchKernelGGL(layernorm_wave<NV>, dim3((unsigned)((rows + 3) / 4)), block, 0, s, x, in_row_map, gamma, beta, y, (int)rows, width, eps, bump_lens, bump_count)
    if (vec && width <= 2048 && rows >= 64) {                 // a prompt's rows: one wave each
        if (width <= 512) EET_LNW(1);
        else if (width <= 1024) EET_LNW(2);
        else EET_LNW(4);
    } else if (vec && width <= 2048) EET_LN(1);
    else if (vec && width <= 4096) EET_LN(2);
    else if (vec && width <= 8192) EET_LN(4);
    else if (vec && width <= 16384) EET_LN(8);
    else
        hipLaunchKernelGGL(layernorm_generic, grid, block, 0, s, x, in_row_map, gamma, beta, y, width, eps,
                           bump_lens, bump_count);
#undef EET_LN
#undef EET_LNW
    return hipGetLastError();
}

// ============================================================================================
// add-bias + GELU, add-bias + residual   (4*width resp. 6*width bytes per row)
// ============================================================================================
// grid = (column chunks, row groups); each thread handles one 8-wide vector of a row.
template <bool RES>
__global__ __launch_bounds__(256) void bias_act_vec(const half_t* __restrict__ x, const half_t* __restrict__ bias,
                                                    const half_t* __restrict__ res, half_t* __restrict__ y,
                                                    int64_t rows, int width) {
    const int nvec = width >> 3;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= nvec) return;
    const half8v b = reinterpret_cast<const half8v*>(bias)[c];
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const int64_t off = r * nvec + c;
        const half8v v = reinterpret_cast<const half8v*>(x)[off];
        half8v o;
        if (RES) {
            const half8v rr = reinterpret_cast<const half8v*>(res)[off];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (half_t)((float)v[e] + (float)b[e] + (float)rr[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (half_t)gelu_tanh((float)v[e] + (float)b[e]);
        }
        reinterpret_cast<half8v*>(y)[off] = o;
    }
}

template <bool RES>
__global__ __launch_bounds__(256) void bias_act_scalar(const half_t* __restrict__ x, const half_t* __restrict__ bias,
                                                       const half_t* __restrict__ res, half_t* __restrict__ y,
                                                       int64_t rows, int width) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= width) return;
    const float b = (float)bias[c];
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const int64_t off = r * width + c;
        const float v = (float)x[off] + b;
        y[off] = (half_t)(RES ? v + (float)res[off] : gelu_tanh(v));
    }
}

template <bool RES>
static hipError_t launch_bias_act(const half_t* x, const half_t* bias, const half_t* res, half_t* y,
                                  int64_t rows, int width, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const unsigned gy = (unsigned)(rows < 32768 ? rows : 32768);
    const bool vec = (width % 8 == 0) && aligned16(x) && aligned16(y) && aligned16(bias) && (!RES || aligned16(res));
    if (vec) {
        const dim3 grid((width / 8 + 255) / 256, gy);
        hipLaunchKernelGGL(bias_act_vec<RES>, grid, dim3(256), 0, s, x, bias, res, y, rows, width);
    } else {
        const dim3 grid((width + 255) / 256, gy);
        hipLaunchKernelGGL(bias_act_scalar<RES>, grid, dim3(256), 0, s, x, bias, res, y, rows, width);
    }
    return hipGetLastError();
}

hipError_t launch_bias_gelu(const half_t* x, const half_t* bias, half_t* y, int64_t rows, int width, hipStream_t s) {
    return launch_bias_act<false>(x, bias, nullptr, y, rows, width, s);
}
hipError_t launch_bias_residual(const half_t* x, const half_t* bias, const half_t* res, half_t* y, int64_t rows,
                                int width, hipStream_t s) {
    return launch_bias_act<true>(x, bias, res, y, rows, width, s);
}

// ============================================================================================
// Mask-free softmax (Algorithm 1), in place on scores [batch, heads, S, S]
// ============================================================================================
// One wave per query row.  Row i of sequence b is visited only if i < len[b] (pad queries are
// skipped); its window is keys 0..i -- the comparison of key index against query index that
// replaces the attention mask -- and entries i+1..S-1 of a visited row are set to zero.
// NV = 8-wide vectors cached per lane (S <= NV*512, S % 8 == 0).
template <int NV>
__global__ __launch_bounds__(256) void softmax_maskfree_vec(half_t* __restrict__ scores, SeqLens lens, int heads,
                                                            int S, float scale_log2e, int left) {
    const int lane = threadIdx.x % kWave;
    const int i = blockIdx.x * 4 + threadIdx.x / kWave;   // query row
    const int bh = blockIdx.y;
    const int b = bh / heads;
    const int first = left ? S - lens.len[b] : 0;          // Algorithm 1's padLen when the pads lead: first non-pad position
    if (i < first || i >= first + lens.len[b]) return;     // pad rows; also covers i >= S
    half8v* row = reinterpret_cast<half8v*>(scores + ((size_t)bh * S + i) * S);
    const int nvec = S >> 3;
    const int nwin = (i >> 3) + 1;                         // vectors up to the end of the window first..i
    const int vwin = first >> 3;                           // ... and from its start

    float t[NV][8];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int idx = lane + c * kWave;
        if (idx >= vwin && idx < nwin) {
            const half8v v = row[idx];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = idx * 8 + e <= i && idx * 8 + e >= first;
                t[c][e] = ok ? (float)v[e] * scale_log2e : -INFINITY;
                m = fmaxf(m, t[c][e]);
            }
        }
    }
    m = wave_max(m);                                       // the first key is always in the window: m is finite
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int idx = lane + c * kWave;
        if (idx >= vwin && idx < nwin) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                t[c][e] = exp2f(t[c][e] - m);              // exp2(-inf) = 0 for masked entries
                sum += t[c][e];
            }
        }
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int idx = lane + c * kWave;
        if (idx < nvec) {
            half8v o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (idx >= vwin && idx < nwin) ? (half_t)(t[c][e] * inv) : (half_t)0.f;
            row[idx] = o;
        }
    }
}

// Any S: scalar three-pass version, one wave per row.
__global__ __launch_bounds__(256) void softmax_maskfree_generic(half_t* __restrict__ scores, SeqLens lens,
                                                                int heads, int S, float scale_log2e, int left) {
    const int lane = threadIdx.x % kWave;
    const int i = blockIdx.x * 4 + threadIdx.x / kWave;
    const int bh = blockIdx.y;
    const int b = bh / heads;
    const int first = left ? S - lens.len[b] : 0;
    if (i < first || i >= first + lens.len[b]) return;
    half_t* row = scores + ((size_t)bh * S + i) * S;
    float m = -INFINITY;
    for (int j = first + lane; j <= i; j += kWave) m = fmaxf(m, (float)row[j] * scale_log2e);
    m = wave_max(m);
    float sum = 0.f;
    for (int j = first + lane; j <= i; j += kWave) sum += exp2f((float)row[j] * scale_log2e - m);
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
    for (int j = lane; j < S; j += kWave)
        row[j] = (j >= first && j <= i) ? (half_t)(exp2f((float)row[j] * scale_log2e - m) * inv) : (half_t)0.f;
}

hipError_t launch_softmax_maskfree(half_t* scores, const SeqLens& lens, int batch, int heads, int S, float scale,
                                   hipStream_t s, bool left_padded) {
    const int left = left_padded ? 1 : 0;
    const dim3 grid((S + 3) / 4, batch * heads), block(256);
    const float sl2 = scale * 1.4426950408889634f;
    const bool vec = (S % 8 == 0) && aligned16(scores);
#define EET_SM(NV) hipLaunchKernelGGL(softmax_maskfree_vec<NV>, grid, block, 0, s, scores, lens, heads, S, sl2, left)
    if (vec && S <= 512) EET_SM(1);
    else if (vec && S <= 1024) EET_SM(2);
    else if (vec && S <= 2048) EET_SM(4);
    else if (vec && S <= 4096) EET_SM(8);
    else if (vec && S <= 8192) EET_SM(16);
    else hipLaunchKernelGGL(softmax_maskfree_generic, grid, block, 0, s, scores, lens, heads, S, sl2, left);
#undef EET_SM
    return hipGetLastError();
}

// ============================================================================================
// Prefill index set-up: the padding offsets become integers on the device, nothing else.
// ============================================================================================
// One block per padded row r = b*S + i.  Valid row: record packed->padded map.  Pad row: zero
// the output row.  Block 0 also publishes the lengths and their prefix sums.
__global__ __launch_bounds__(64) void prefill_setup(SeqLens lens, int batch, int S, int width,
                                                    int32_t* __restrict__ cache_lens, int32_t* __restrict__ cu_seqlens,
                                                    int32_t* __restrict__ row_map, half_t* __restrict__ out, int left) {
    const int r = blockIdx.x;
    const int b = r / S, i = r % S;
    int cu = 0;
    for (int k = 0; k < b; ++k) cu += lens.len[k];
    const int first = left ? S - lens.len[b] : 0;          // position of the sequence's token 0 in its padded row block
    if (i >= first && i < first + lens.len[b]) {
        if (threadIdx.x == 0) row_map[cu + i - first] = r;
    } else {
        half_t* o = out + (size_t)r * width;
        if ((width & 7) == 0) {
            half8v z;
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = (half_t)0.f;
            for (int c = threadIdx.x; c < (width >> 3); c += 64) reinterpret_cast<half8v*>(o)[c] = z;
        } else {
            for (int c = threadIdx.x; c < width; c += 64) o[c] = (half_t)0.f;
        }
    }
    if (r == 0) {
        int acc = 0;
        for (int k = threadIdx.x; k < batch; k += 64) cache_lens[k] = lens.len[k];
        if (threadIdx.x == 0) {
            for (int k = 0; k < batch; ++k) {
                cu_seqlens[k] = acc;
                acc += lens.len[k];
            }
            cu_seqlens[batch] = acc;
        }
    }
}

// The device-side cache lengths set from the host (resuming from a saved K/V cache): one small fill kernel, so the
// call can sit in a stream or a captured graph like every other.
__global__ __launch_bounds__(kMaxBatch) void set_cache_lens(SeqLens lens, int batch, int32_t* __restrict__ cache_lens) {
    if ((int)threadIdx.x < batch) cache_lens[threadIdx.x] = lens.len[threadIdx.x];
}

hipError_t launch_set_cache_lens(const SeqLens& lens, int batch, int32_t* cache_lens, hipStream_t s) {
    hipLaunchKernelGGL(set_cache_lens, dim3(1), dim3(kMaxBatch), 0, s, lens, batch, cache_lens);
    return hipGetLastError();
}

hipError_t launch_prefill_setup(const SeqLens& lens, int batch, int S, int width, int32_t* cache_lens,
                                int32_t* cu_seqlens, int32_t* row_map, half_t* out, hipStream_t s, bool left_padded) {
    hipLaunchKernelGGL(prefill_setup, dim3(batch * S), dim3(64), 0, s, lens, batch, S, width, cache_lens,
                       cu_seqlens, row_map, out, left_padded ? 1 : 0);
    return hipGetLastError();
}

}  // namespace eet
