// Dense projections y = x W^T + b with fused epilogues (QKV scatter into the K/V cache,
// add-bias+GELU, add-bias+residual with optional row scatter back to the padded layout).
//
// The paper leaves these to library GEMM calls followed by separate bias/activation kernels
// (Section 3.2: "kernels are not always fused, especially ... GEMM calls").  Here the epilogue
// runs on the accumulators, so the intermediate never visits HBM.
//
// Two kernels:
//   gemm_mfma    prefill (M = valid tokens of the batch, packed): LDS-tiled, v_mfma_f32_32x32x16_f16,
//                double-buffered LDS with register prefetch; bound by the matrix cores.
//   gemm_skinny  decode (M <= 16 rows): every weight is read from HBM exactly once per step, so the
//                kernel is a weight stream; v_mfma_f32_16x16x32_f16 does the 16-row contraction on
//                fragments loaded straight from global memory, K is split over the 4 waves of a
//                workgroup and reduced through LDS.
// Both compute the transposed tile (weights as the MFMA "A" operand) so that each lane ends up
// with 4 consecutive output columns of one row: 8-byte stores, and 8-byte bias/residual loads.
#include <cstdlib>

#include "kernels.hpp"

namespace eet {

// --------------------------------------------------------------------------------------------
// epilogue on 4 consecutive output columns n..n+3 of row m
// --------------------------------------------------------------------------------------------
template <int EPI>
__device__ __forceinline__ void epilogue4(const GemmArgs& a, int m, int n, float v0, float v1, float v2, float v3) {
    const half4v b = *reinterpret_cast<const half4v*>(a.bias + n);
    v0 += (float)b[0]; v1 += (float)b[1]; v2 += (float)b[2]; v3 += (float)b[3];
    if (EPI == EPI_BIAS_GELU) {
        v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3);
    }
    if (EPI == EPI_BIAS_RES) {
        const int64_t rr = a.res_row_map ? (int64_t)a.res_row_map[m] : (int64_t)m;
        const half4v r = *reinterpret_cast<const half4v*>(a.res + rr * a.N + n);
        v0 += (float)r[0]; v1 += (float)r[1]; v2 += (float)r[2]; v3 += (float)r[3];
    }
    half4v o;
    o[0] = (half_t)v0; o[1] = (half_t)v1; o[2] = (half_t)v2; o[3] = (half_t)v3;
    if (EPI == EPI_QKV) {
        const int which = n / a.hidden;          // 0 = Q, 1 = K, 2 = V
        const int c = n - which * a.hidden;
        if (which == 0) {
            *reinterpret_cast<half4v*>(a.y + (int64_t)m * a.hidden + c) = o;
        } else {
            int b_, pos;
            if (a.tok_row_map) {                 // prefill: token -> (sequence, position)
                const int r = a.tok_row_map[m];
                b_ = r / a.S;
                pos = r - b_ * a.S;
            } else {                             // decode: the new token goes to slot n_b
                b_ = m;
                pos = a.lens[m];
            }
            const int g = c / a.d, dd = c - g * a.d;
            half_t* cache = which == 1 ? a.k_cache : a.v_cache;
            *reinterpret_cast<half4v*>(cache + (((int64_t)b_ * a.heads + g) * a.max_seq + pos) * a.d + dd) = o;
        }
        return;
    }
    const int64_t orow = a.out_row_map ? (int64_t)a.out_row_map[m] : (int64_t)m;
    *reinterpret_cast<half4v*>(a.y + orow * a.N + n) = o;
}

// --------------------------------------------------------------------------------------------
// MFMA tile kernel
// --------------------------------------------------------------------------------------------
constexpr int kBK = 64;          // K depth of one LDS stage
constexpr int kLdk = kBK + 8;    // padded LDS row (144 B): 16-byte fragment reads hit distinct banks

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_mfma(GemmArgs a, int tiles_m, int tiles_n) {
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;       // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;         // 32x32 fragments per wave
    constexpr int AV = BM * 8 / NT, WV = BN * 8 / NT; // 16-byte vectors each thread stages per K step
    static_assert(AV >= 1 && WV >= 1 && WM % 32 == 0 && WN % 32 == 0, "tile shape");

    __shared__ __attribute__((aligned(16))) half_t As[2][BM * kLdk];
    __shared__ __attribute__((aligned(16))) half_t Ws[2][BN * kLdk];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of tiles
    // so that neighbours in the range (which share a weight panel) also share an L2.
    const int nb = tiles_m * tiles_n;
    const int pid = blockIdx.x;
    const int xcd = pid & 7, local = pid >> 3;
    const int q = nb >> 3, rem = nb & 7;
    const int tile = xcd * q + (xcd < rem ? xcd : rem) + local;
    const int tile_n = tile / tiles_m, tile_m = tile - tile_n * tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int M = a.M, N = a.N, K = a.K;

    half8v ra[AV], rw[WV];
    auto gload = [&](int kt) {
#pragma unroll
        for (int v = 0; v < AV; ++v) {
            const int idx = tid + v * NT, row = idx >> 3, ch = idx & 7;
            int gr = m0 + row;
            gr = gr < M ? gr : M - 1;                                  // rows past the tail: clamp, never stored
            ra[v] = *reinterpret_cast<const half8v*>(a.x + (int64_t)gr * K + kt * kBK + ch * 8);
        }
#pragma unroll
        for (int v = 0; v < WV; ++v) {
            const int idx = tid + v * NT, row = idx >> 3, ch = idx & 7;
            int gr = n0 + row;
            gr = gr < N ? gr : N - 1;
            rw[v] = *reinterpret_cast<const half8v*>(a.w + (int64_t)gr * K + kt * kBK + ch * 8);
        }
    };
    auto sstore = [&](int st) {
#pragma unroll
        for (int v = 0; v < AV; ++v) {
            const int idx = tid + v * NT, row = idx >> 3, ch = idx & 7;
            *reinterpret_cast<half8v*>(&As[st][row * kLdk + ch * 8]) = ra[v];
        }
#pragma unroll
        for (int v = 0; v < WV; ++v) {
            const int idx = tid + v * NT, row = idx >> 3, ch = idx & 7;
            *reinterpret_cast<half8v*>(&Ws[st][row * kLdk + ch * 8]) = rw[v];
        }
    };

    float16v acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = K / kBK;
    gload(0);
    sstore(0);
    __syncthreads();
    const int frow = lane & 31, fk = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        if (kt + 1 < nk) gload(kt + 1);
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            half8v fa[FM], fw[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                fa[i] = *reinterpret_cast<const half8v*>(&As[st][(wm0 + i * 32 + frow) * kLdk + ks * 16 + fk]);
#pragma unroll
            for (int j = 0; j < FN; ++j)
                fw[j] = *reinterpret_cast<const half8v*>(&Ws[st][(wn0 + j * 32 + frow) * kLdk + ks * 16 + fk]);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) sstore(st ^ 1);
        __syncthreads();
    }

    // acc[i][j][r]: row m = lane%32 of fragment i, column n = (r/4)*8 + (lane/32)*4 + r%4 of fragment j
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm0 + i * 32 + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n = n0 + wn0 + j * 32 + rg * 8 + (lane >> 5) * 4;
                if (n < N)
                    epilogue4<EPI>(a, m, n, acc[i][j][rg * 4 + 0], acc[i][j][rg * 4 + 1], acc[i][j][rg * 4 + 2],
                                   acc[i][j][rg * 4 + 3]);
            }
        }
    }
}

// --------------------------------------------------------------------------------------------
// weight-streaming kernel for M <= 16 rows per grid.y slice
// --------------------------------------------------------------------------------------------
// Workgroup = 4 waves; it owns 16*NF output columns.  K steps of 32 are dealt round-robin to
// the waves (adjacent waves read adjacent 64-byte pieces of the same weight rows).
template <int NF, int EPI>
__global__ __launch_bounds__(256) void gemm_skinny(GemmArgs a) {
    constexpr int UN = 4;                       // K steps in flight per wave
    __shared__ float red[4][NF * 16][17];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, G = lane >> 4;
    const int n0 = blockIdx.x * (NF * 16), mc = blockIdx.y * 16;
    const int M = a.M, N = a.N, K = a.K;
    const int nsteps = K / 32;

    int xr = mc + fr;
    xr = xr < M ? xr : M - 1;
    const half_t* xp = a.x + (int64_t)xr * K + G * 8;
    const half_t* wp[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int wr = n0 + f * 16 + fr;
        wr = wr < N ? wr : N - 1;
        wp[f] = a.w + (int64_t)wr * K + G * 8;
    }
    float4v acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) acc[f] = float4v{0.f, 0.f, 0.f, 0.f};

    for (int s0 = wave; s0 < nsteps; s0 += 4 * UN) {
        half8v xf[UN], wf[UN][NF];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int step = s0 + 4 * u;
            const bool ok = step < nsteps;
            const int k = (ok ? step : s0) * 32;
            xf[u] = *reinterpret_cast<const half8v*>(xp + k);
            if (!ok) {
#pragma unroll
                for (int e = 0; e < 8; ++e) xf[u][e] = (half_t)0.f;
            }
#pragma unroll
            for (int f = 0; f < NF; ++f) wf[u][f] = *reinterpret_cast<const half8v*>(wp[f] + k);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u)
#pragma unroll
            for (int f = 0; f < NF; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[u][f], xf[u], acc[f], 0, 0, 0);
    }
    // acc[f][r]: output column n0 + f*16 + 4G + r, row mc + lane%16
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][f * 16 + 4 * G + r][fr] = acc[f][r];
    __syncthreads();
    for (int t = tid; t < 64 * NF; t += 256) {
        const int ng = t % (4 * NF), ml = t / (4 * NF);
        const int m = mc + ml, n = n0 + ng * 4;
        if (m >= M || n >= N) continue;
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            v[c] = red[0][ng * 4 + c][ml] + red[1][ng * 4 + c][ml] + red[2][ng * 4 + c][ml] + red[3][ng * 4 + c][ml];
        epilogue4<EPI>(a, m, n, v[0], v[1], v[2], v[3]);
    }
}

// --------------------------------------------------------------------------------------------
// dispatch
// --------------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN>
static void launch_mfma_cfg(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const int tm = (a.M + BM - 1) / BM, tn = (a.N + BN - 1) / BN;
    const dim3 grid(tm * tn), block(WGM * WGN * 64);
    switch (epi) {
        case EPI_BIAS: hipLaunchKernelGGL((gemm_mfma<BM, BN, WGM, WGN, EPI_BIAS>), grid, block, 0, s, a, tm, tn); break;
        case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_mfma<BM, BN, WGM, WGN, EPI_BIAS_GELU>), grid, block, 0, s, a, tm, tn); break;
        case EPI_BIAS_RES: hipLaunchKernelGGL((gemm_mfma<BM, BN, WGM, WGN, EPI_BIAS_RES>), grid, block, 0, s, a, tm, tn); break;
        case EPI_QKV: hipLaunchKernelGGL((gemm_mfma<BM, BN, WGM, WGN, EPI_QKV>), grid, block, 0, s, a, tm, tn); break;
    }
}

template <int NF>
static void launch_skinny_cfg(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const dim3 grid((a.N + NF * 16 - 1) / (NF * 16), (a.M + 15) / 16), block(256);
    switch (epi) {
        case EPI_BIAS: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS>), grid, block, 0, s, a); break;
        case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS_GELU>), grid, block, 0, s, a); break;
        case EPI_BIAS_RES: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS_RES>), grid, block, 0, s, a); break;
        case EPI_QKV: hipLaunchKernelGGL((gemm_skinny<NF, EPI_QKV>), grid, block, 0, s, a); break;
    }
}

hipError_t launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    if (a.M <= 0) return hipSuccess;
    if (a.M <= 16) {
        // enough workgroups to cover the chip first, then wider slices to amortise the activations
        if (a.N >= 64 * 1024) launch_skinny_cfg<4>(a, epi, s);
        else if (a.N >= 32 * 1024) launch_skinny_cfg<2>(a, epi, s);
        else launch_skinny_cfg<1>(a, epi, s);
    } else {
        static const int tile = getenv("EET_GEMM_TILE") ? atoi(getenv("EET_GEMM_TILE")) : 0;
        switch (tile) {
            case 1: launch_mfma_cfg<256, 256, 2, 2>(a, epi, s); break;
            case 2: launch_mfma_cfg<256, 256, 2, 4>(a, epi, s); break;
            case 3: launch_mfma_cfg<256, 128, 2, 2>(a, epi, s); break;
            case 4: launch_mfma_cfg<256, 128, 4, 2>(a, epi, s); break;
            default: launch_mfma_cfg<128, 128, 2, 2>(a, epi, s); break;
        }
    }
    return hipGetLastError();
}

}  // namespace eet
