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

// tanh-form GELU in fp32 (the GPT-2 activation): 0.5 x (1 + tanh(u)), u = sqrt(2/pi) (x + 0.044715 x^3), written as
// x * sigmoid(2u) = x / (1 + 2^(-x (A + B x^2))) with A = 2 sqrt(2/pi) log2(e), B = 0.044715 A: seven vector
// instructions (one v_exp_f32, one v_rcp_f32), exact limits at +-inf (x * 0 and x * 1), no cancellation.
__device__ __forceinline__ float gelu_tanh(float x) {
    constexpr float A = 2.3022081985f, B = 0.10294323952f;
    const float t = __builtin_fmaf(x * x, B, A);
    const float e = __builtin_amdgcn_exp2f(-x * t);
    return x * __builtin_amdgcn_rcpf(e + 1.0f);
}

}  // namespace eet
