// Shared device-side vocabulary for the gfx950 kernels: vector types, wave64 reductions,
// fp16 <-> fp32 helpers.  Everything here is inline device code; no host logic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace eet {

typedef _Float16 half_t;
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;  // CDNA wavefront width

// Per-sequence lengths of one call, passed by value as a kernel argument (the only
// host->device metadata of a prefill: no mask tensor exists, Section 2.1 of the paper).
constexpr int kMaxBatch = 128;
struct SeqLens {
    int32_t len[kMaxBatch];
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Sum over a workgroup of NW waves; every thread gets the result.  `red` is LDS scratch of
// at least NW floats, reusable after the call returns.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    if (NW == 1) return v;
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    __syncthreads();
    if (l == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    return t;
}

// Load of data that a launch reads once (the weights of a decode step, the K/V rows of a decode attention): the
// non-temporal hint.  A read-only stream of 1-2 GB runs at 6.6-6.9 TB/s with it and at 5.5-6.05 TB/s without (16-byte
// loads, 8 or 16 in flight per lane, any grid), and the decode kernels gain the same tenth: cfg5b's attention 202 -> 180
// us, its FFN-2 weight stream 206 -> 187 us.  Operands that other workgroups read again (activation rows) keep plain loads.
template <class T>
__device__ __forceinline__ T load_once(const T* p) {
    return __builtin_nontemporal_load(p);
}

// tanh-form GELU in fp32 (the GPT-2 activation): 0.5 x (1 + tanh(u)), u = sqrt(2/pi) (x + 0.044715 x^3), written as
// x * sigmoid(2u) = x / (1 + 2^(-x (A + B x^2))) with A = 2 sqrt(2/pi) log2(e), B = 0.044715 A: seven vector
// instructions (one v_exp_f32, one v_rcp_f32), exact limits at +-inf (x * 0 and x * 1), no cancellation.
__device__ __forceinline__ float gelu_tanh(float x) {
    constexpr float A = 2.3022081985f, B = 0.10294323952f;
    const float t = __builtin_fmaf(x * x, B, A);
    const float e = __builtin_amdgcn_exp2f(-x * t);
    return x * __builtin_amdgcn_rcpf(e + 1.0f);
}

// The work of one prefetch workgroup (see PrefetchArgs in kernels.hpp): part `part` of `parts`, `nthreads` threads.
// One 4-byte load per 128-byte line.  The loads are ordinary loads whose values are xor-ed into a register that an
// empty asm statement "uses" at the end: nothing is stored, the compiler cannot drop the loads, and it keeps track
// of the registers they land in (a load whose destination the compiler believes dead would write that register
// later, after it has been given to something else).
// lines [lo, hi) of `base`, thread tid of nthreads: eight independent loads in flight per thread
__device__ __forceinline__ int touch_lines(const char* base, uint32_t lo, uint32_t hi, int tid, int nthreads) {
    int acc = 0;
    for (uint32_t i = lo + tid; i < hi; i += 8u * nthreads) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t j = i + (uint32_t)u * nthreads;
            v[u] = j < hi ? *reinterpret_cast<const int*>(base + (size_t)j * 128) : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    return acc;
}
template <class PF>
__device__ __forceinline__ void run_prefetch(const PF& p, int part, int parts, int tid, int nthreads) {
    int acc = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const uint32_t lines = p.lin_lines[r];
        const uint32_t per = (lines + parts - 1) / parts, lo = part * per;
        const uint32_t hi = lo + per < lines ? lo + per : lines;
        if (lo < hi) acc ^= touch_lines(static_cast<const char*>(p.lin[r]), lo, hi, tid, nthreads);
    }
    if (p.k_cache != nullptr) {
        const int pairs = p.kv_batch * p.kv_heads;
        for (int bh = part; bh < pairs; bh += parts) {
            int rows = p.lens[bh / p.kv_heads];
            rows = rows < 0 ? 0 : (rows > p.kv_capacity ? p.kv_capacity : rows);                  // never past the pair's slots
            const uint32_t lines = (uint32_t)rows * (uint32_t)(p.kv_d * 2 / 128);                  // a row is 128 or 256 bytes
            const size_t off = (size_t)bh * p.kv_capacity * p.kv_d * 2;
            acc ^= touch_lines(reinterpret_cast<const char*>(p.k_cache) + off, 0, lines, tid, nthreads);
            acc ^= touch_lines(reinterpret_cast<const char*>(p.v_cache) + off, 0, lines, tid, nthreads);
        }
    }
    asm volatile("" ::"v"(acc));
}

}  // namespace eet
