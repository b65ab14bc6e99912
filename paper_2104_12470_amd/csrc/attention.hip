// Mask-free multi-head attention for gfx950: whole-prompt (prefill) and incremental (decode).
//
// Mask fusion (Section 2.1, Algorithm 1): the causal mask is the comparison "key index <= query
// index" evaluated on the lane's own indices, and the padding mask is the loop bound -- key
// tiles beyond the query tile or beyond the sequence's valid length are never loaded, query
// tiles of pad rows are never scheduled.  Unlike Algorithm 1, the scores are not materialised:
// QK^T, the windowed softmax and PV are one kernel with an online softmax, so row length is
// unbounded (the goal of Section 2.2) and the S x S buffer of Section 3.2 is not needed.
//
// K/V cache layout: [batch][heads][capacity][d] fp16, slot t = token t of the sequence.
#include <cstdlib>
#include "kernels.hpp"

namespace eet {

constexpr float kLog2e = 1.4426950408889634f;

// ============================================================================================
// Prefill: flash-style, v_mfma_f32_32x32x16_f16
// ============================================================================================
// Workgroup = 4 waves = 128 query rows of one (sequence, head); wave w owns rows 32w..32w+31.
// Key tiles of 64 are staged through LDS: K row-major, V transposed (so that both MFMA operands
// of P.V read 8-byte runs along the key axis).  The kernel computes S^T = K Q^T, which leaves
// every lane holding scores of ONE query (column lane%32): row statistics need a single
// cross-lane exchange (lane ^ 32) and P^T is already in MFMA B-operand layout for
// O^T = V^T P^T.
template <int D>
__global__ __launch_bounds__(256, 2) void attn_prefill(AttnPrefillArgs a, SeqLens lens) {
    constexpr int BQ = 128, BKV = 64;
    constexpr int LDKS = D + 8;         // K tile row stride (halfs): 16-byte reads conflict-free
    constexpr int LDVT = BKV + 8;       // V^T tile row stride
    constexpr int KVEC = BKV * D / 8 / 256;   // 16-byte vectors of K per thread per tile
    constexpr int RPT = D / 32;               // V rows per thread per tile (transposed on the way to LDS)
    constexpr int DCH = D / 8;                // 16-byte chunks per K/V row
    __shared__ __attribute__((aligned(16))) half_t Ks[BKV * LDKS];
    __shared__ __attribute__((aligned(16))) half_t Vt[D * LDVT];

    const int b = blockIdx.z, g = blockIdx.y;
    const int L = lens.len[b];
    const int i0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * BQ;   // longest (latest) query tiles first
    if (i0 >= L) return;                                          // pad queries are never visited
    int row0 = b * a.S;
    if (a.packed) {
        row0 = 0;
        for (int k = 0; k < b; ++k) row0 += lens.len[k];
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, G = lane >> 5;
    const int iw0 = i0 + wave * 32;
    const int i = iw0 + li;                  // this lane's query position
    const bool row_ok = i < L;

    // Q^T fragments (B operand): column i, depth kk*16 + G*8 .. +8
    half8v qf[D / 16];
    {
        const half_t* qp = a.q + (int64_t)(row0 + (row_ok ? i : L - 1)) * a.hidden + g * D + G * 8;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) qf[kk] = *reinterpret_cast<const half8v*>(qp + kk * 16);
    }
    const int64_t head_off = ((int64_t)b * a.heads + g) * a.capacity * D;
    const half_t* kbase = a.k_cache + head_off;
    const half_t* vbase = a.v_cache + head_off;

    float16v o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float c = rsqrtf((float)D) * kLog2e;

    const int jlast = (i0 + BQ - 1 < L - 1) ? i0 + BQ - 1 : L - 1;   // last key any row of the tile sees
    const int ntiles = jlast / BKV + 1;

    half8v rk[KVEC], rv[RPT];
    const int v_jg = tid % (BKV / RPT), v_dc = tid / (BKV / RPT);
    auto gload = [&](int jt) {
        const int j0 = jt * BKV;
#pragma unroll
        for (int v = 0; v < KVEC; ++v) {
            const int idx = tid + v * 256, row = idx / DCH, ch = idx % DCH;
            int jr = j0 + row;
            jr = jr < L ? jr : L - 1;        // slots >= L are never read (they may hold anything)
            rk[v] = *reinterpret_cast<const half8v*>(kbase + (int64_t)jr * D + ch * 8);
        }
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            int jr = j0 + v_jg * RPT + r;
            jr = jr < L ? jr : L - 1;
            rv[r] = *reinterpret_cast<const half8v*>(vbase + (int64_t)jr * D + v_dc * 8);
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int v = 0; v < KVEC; ++v) {
            const int idx = tid + v * 256, row = idx / DCH, ch = idx % DCH;
            *reinterpret_cast<half8v*>(&Ks[row * LDKS + ch * 8]) = rk[v];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            half_t* dst = &Vt[(v_dc * 8 + e) * LDVT + v_jg * RPT];
            if (RPT == 4) {
                half4v t;
                t[0] = rv[0][e]; t[1] = rv[1][e]; t[2] = rv[2 % RPT][e]; t[3] = rv[3 % RPT][e];
                *reinterpret_cast<half4v*>(dst) = t;
            } else {
                half2v t;
                t[0] = rv[0][e]; t[1] = rv[1][e];
                *reinterpret_cast<half2v*>(dst) = t;
            }
        }
    };

    gload(0);
    for (int jt = 0; jt < ntiles; ++jt) {
        __syncthreads();                     // everyone is done reading the previous tile
        sstore();
        __syncthreads();
        if (jt + 1 < ntiles) gload(jt + 1);  // in flight during the MFMAs below
        const int j0 = jt * BKV;
        if (j0 > iw0 + 31) continue;         // whole key tile is in the future of this wave's rows

        // S^T[j][i] for 64 keys x 32 queries
        float16v st[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) st[jb][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                const half8v kf = *reinterpret_cast<const half8v*>(&Ks[(jb * 32 + li) * LDKS + kk * 16 + G * 8]);
                st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[kk], st[jb], 0, 0, 0);
            }
        }
        // st[jb][r] belongs to key j0 + jb*32 + (r/4)*8 + G*4 + r%4 and query i.
        // The attention mask is an index comparison, and only tiles that straddle the diagonal of
        // this wave's rows pay for it (wave-uniform branch).
        float tmax = -INFINITY;
        if (j0 + BKV - 1 > iw0) {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + jb * 32 + (r >> 2) * 8 + G * 4 + (r & 3);
                    if (j > i) st[jb][r] = -INFINITY;
                    tmax = fmaxf(tmax, st[jb][r]);
                }
        } else {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, st[jb][r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
        // running maximum m lives in the exp2 domain (score * c): p = 2^(s*c - m), one FMA + one v_exp_f32
        const float m_new = fmaxf(m, tmax * c);      // finite: key 0 is visible to every row
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float psum = 0.f;
        half8v pf[2][2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][r], c, -m_new));
                psum += p;
                pf[jb][r >> 3][r & 7] = (half_t)p;
            }
        l = l * alpha + psum;
        m = m_new;
        if (__any(alpha != 1.0f)) {                  // the maximum stops moving after the first tiles of a long row
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        }
        // O^T[dv][i] += V^T[dv][j] P^T[j][i]; operand slot s of lane group G <-> key
        // jb*32 + hf*16 + (s/4)*8 + G*4 + s%4 (the keys this lane already holds in pf[jb][hf]).
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const half_t* vp = &Vt[(db * 32 + li) * LDVT + jb * 32 + hf * 16 + G * 4];
                    const half4v lo = *reinterpret_cast<const half4v*>(vp);
                    const half4v hi = *reinterpret_cast<const half4v*>(vp + 8);
                    half8v vf;
                    vf[0] = lo[0]; vf[1] = lo[1]; vf[2] = lo[2]; vf[3] = lo[3];
                    vf[4] = hi[0]; vf[5] = hi[1]; vf[6] = hi[2]; vf[7] = hi[3];
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[jb][hf], o[db], 0, 0, 0);
                }
    }

    l += __shfl_xor(l, 32, kWave);
    if (!row_ok) return;
    const float inv = 1.0f / l;
    half_t* op = a.ctx + (int64_t)(row0 + i) * a.hidden + g * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            half4v t;
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = (half_t)(o[db][rg * 4 + e] * inv);
            *reinterpret_cast<half4v*>(op + db * 32 + rg * 8 + G * 4) = t;
        }
}

hipError_t launch_attention_prefill(const AttnPrefillArgs& a, const SeqLens& lens, hipStream_t s) {
    const dim3 grid((a.max_len + 127) / 128, a.heads, a.batch), block(256);
    if (a.d == 128) hipLaunchKernelGGL(attn_prefill<128>, grid, block, 0, s, a, lens);
    else hipLaunchKernelGGL(attn_prefill<64>, grid, block, 0, s, a, lens);
    return hipGetLastError();
}

// ============================================================================================
// Decode: one query per (sequence, head), K and V streamed once from HBM
// ============================================================================================
// grid = (splits, heads, batch); a workgroup of 4 waves owns one contiguous range of keys, each
// wave a quarter of it, walked in chunks of 64 keys whose loads are all issued before any of them
// is used (the work per (sequence, head) is small: memory-level parallelism, not arithmetic, sets
// the speed).  Per group of 16 keys the K fragments go straight from global memory into
// v_mfma_f32_16x16x32_f16 (the query replicated over the 16 columns), so the q.k reduction costs
// no cross-lane traffic; every lane of group G = lane/16 then holds the scores of keys 4G..4G+3
// and multiplies them into its own 16-byte slice of those keys' V rows.
// The padding offset is the loop bound: slots >= n_b are never read.
//
// With more than one range per (sequence, head) each workgroup writes a partial (max, sum,
// values) and attn_decode_combine merges them.
template <int D>
__global__ __launch_bounds__(256) void attn_decode(AttnDecodeArgs a) {
    constexpr int CH = D / 8;            // 16-byte chunks per row (16 or 8)
    constexpr int VR = CH == 16 ? 4 : 2; // V rows per lane per group of 16 keys
    constexpr int KF = D / 32;           // K fragments per group
    constexpr int U = 4;                 // groups in flight per wave
    __shared__ float sm_m[4], sm_l[4];
    __shared__ float sm_acc[4][D];

    const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, G = lane >> 4;
    const int n = a.lens[b] + a.len_bias;                // visible keys
    const int splits = a.splits;
    int per = (n + splits - 1) / splits;
    per = (per + 15) & ~15;
    const int c0 = sp * per;
    const int c1 = (c0 + per < n) ? c0 + per : n;        // may be <= c0: empty range of a short sequence
    const int64_t bh = (int64_t)b * a.heads + g;
    const half_t* kbase = a.k_cache + bh * a.capacity * D;
    const half_t* vbase = a.v_cache + bh * a.capacity * D;

    // this wave's quarter of the range
    int pw = (c1 - c0 + 3) / 4;
    pw = pw > 0 ? (pw + 15) & ~15 : 0;
    const int w0 = c0 + wave * pw;
    const int w1 = (w0 + pw < c1) ? w0 + pw : c1;

    half8v qf[KF];
#pragma unroll
    for (int kk = 0; kk < KF; ++kk) qf[kk] = *reinterpret_cast<const half8v*>(a.q + bh * D + kk * 32 + G * 8);

    const bool hi = (CH == 8) && fr >= 8;                            // d = 64: lanes 8..15 of a group take rows 4G+2, 4G+3
    const int vc = fr % CH, vr0 = hi ? 2 : 0;                        // V slice of this lane: chunk vc, rows 4G+vr0+r
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    float m = -INFINITY, l = 0.f;
    const float c = rsqrtf((float)D) * kLog2e;

    // One chunk = 16*U keys.  The loads of chunk i+1 are issued before chunk i is consumed (two
    // register buffers, loop unrolled by two); rows past the range are clamped to its last row, so
    // the look-ahead needs no branch and the in-order load counter never waits on the newer chunk.
    auto request = [&](half8v (&kf)[U][KF], half8v (&vf)[U][VR], int j0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int jk = j0 + 16 * u + fr;
            jk = jk < w1 ? jk : w1 - 1;                   // masked in consume()
            jk = jk > 0 ? jk : 0;
#pragma unroll
            for (int kk = 0; kk < KF; ++kk)
                kf[u][kk] = *reinterpret_cast<const half8v*>(kbase + (int64_t)jk * D + kk * 32 + G * 8);
#pragma unroll
            for (int r = 0; r < VR; ++r) {
                int jv = j0 + 16 * u + 4 * G + vr0 + r;
                jv = jv < w1 ? jv : w1 - 1;
                jv = jv > 0 ? jv : 0;
                vf[u][r] = *reinterpret_cast<const half8v*>(vbase + (int64_t)jv * D + vc * 8);
            }
        }
    };
    auto consume = [&](const half8v (&kf)[U][KF], const half8v (&vf)[U][VR], int j0) {
        float t[U][4], gmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float4v s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KF; ++kk) s = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[u][kk], qf[kk], s, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                t[u][r] = (j0 + 16 * u + 4 * G + r < w1) ? s[r] * c : -INFINITY;
                gmax = fmaxf(gmax, t[u][r]);
            }
        }
        gmax = fmaxf(gmax, __shfl_xor(gmax, 16, kWave));
        gmax = fmaxf(gmax, __shfl_xor(gmax, 32, kWave));
        const float m_new = fmaxf(m, gmax);               // finite: key j0 is inside the range
        const float alpha = exp2f(m - m_new);
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) p[r] = exp2f(t[u][r] - m_new);
            l += (p[0] + p[1]) + (p[2] + p[3]);
            // weights of this lane's V rows: rows 4G..4G+3 (d = 128) or the row pair picked by hi (d = 64)
            float pv[VR];
            if (CH == 16) {
#pragma unroll
                for (int r = 0; r < VR; ++r) pv[r] = p[r];
            } else {
                pv[0] = hi ? p[2] : p[0];
                pv[1 % VR] = hi ? p[3] : p[1];
            }
#pragma unroll
            for (int r = 0; r < VR; ++r) {
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += pv[r] * (float)vf[u][r][e];
            }
        }
        m = m_new;
    };
    half8v kA[U][KF], vA[U][VR], kB[U][KF], vB[U][VR];
    if (w0 < w1) {
        request(kA, vA, w0);
        for (int j0 = w0; j0 < w1; j0 += 32 * U) {
            request(kB, vB, j0 + 16 * U);
            __builtin_amdgcn_sched_barrier(0);            // keep the look-ahead loads ahead of the arithmetic
            consume(kA, vA, j0);
            if (j0 + 16 * U >= w1) break;
            request(kA, vA, j0 + 32 * U);
            __builtin_amdgcn_sched_barrier(0);
            consume(kB, vB, j0 + 16 * U);
        }
    }
    // fold the lane groups: keys were spread over G (and over the two row pairs when d = 64)
    l += __shfl_xor(l, 16, kWave);
    l += __shfl_xor(l, 32, kWave);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        acc[e] += __shfl_xor(acc[e], 16, kWave);
        acc[e] += __shfl_xor(acc[e], 32, kWave);
        if (CH == 8) acc[e] += __shfl_xor(acc[e], 8, kWave);
    }
    if (lane < CH) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sm_acc[wave][lane * 8 + e] = acc[e];
    }
    if (lane == 0) {
        sm_m[wave] = m;
        sm_l[wave] = l;
    }
    __syncthreads();
    float M = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));   // -inf only for an empty range
    float Lsum = 0.f, A = 0.f;
    if (tid < D && M > -INFINITY) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = exp2f(sm_m[w] - M);                               // idle wave: exp2(-inf) = 0
            Lsum += sm_l[w] * sc;
            A += sm_acc[w][tid] * sc;
        }
    }
    if (splits == 1) {
        if (tid < D) a.ctx[bh * D + tid] = (half_t)(A / Lsum);
        return;
    }
    if (tid < D) a.part_acc[(bh * splits + sp) * D + tid] = A;
    if (tid == 0) {
        a.part_ml[(bh * splits + sp) * 2 + 0] = M;
        a.part_ml[(bh * splits + sp) * 2 + 1] = Lsum;
    }
}

// Merge the per-range partials (max, sum, weighted values) of the (sequence, head) pairs, in
// range order.  A separate launch: a device-scope release/acquire inside the attention kernel
// (last workgroup merges) costs an L2 write-back and invalidate on this multi-die part, far more
// than the launch it would save.  Workgroup = 256 threads = 256/d pairs; all loads of a pair's
// ranges are issued before they are combined.
template <int D>
__global__ __launch_bounds__(256) void attn_decode_combine(AttnDecodeArgs a) {
    constexpr int PPB = 256 / D;                         // pairs per workgroup
    constexpr int MAXS = 16;                             // ranges held in registers at a time
    const int tid = threadIdx.x, dd = tid % D;
    const int64_t bh = (int64_t)blockIdx.x * PPB + tid / D;
    if (bh >= (int64_t)a.batch * a.heads) return;
    const int splits = a.splits;
    const float* ml = a.part_ml + bh * splits * 2;
    const float* pa = a.part_acc + bh * splits * D + dd;
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[s * 2]);     // range 0 is never empty
    float Lsum = 0.f, A = 0.f;
    for (int s0 = 0; s0 < splits; s0 += MAXS) {
        float mv[MAXS], lv[MAXS], av[MAXS];
#pragma unroll
        for (int u = 0; u < MAXS; ++u) {
            const int s = s0 + u < splits ? s0 + u : splits - 1;
            mv[u] = ml[s * 2];
            lv[u] = ml[s * 2 + 1];
            av[u] = pa[s * D];
        }
#pragma unroll
        for (int u = 0; u < MAXS; ++u) {
            const float sc = s0 + u < splits ? exp2f(mv[u] - M) : 0.f;
            Lsum += lv[u] * sc;
            A += av[u] * sc;
        }
    }
    a.ctx[bh * D + dd] = (half_t)(A / Lsum);
}

int attention_decode_splits(int batch, int heads, int capacity) {
    // One key range per (sequence, head) once there are 128 pairs (measured: as fast as splitting,
    // and no merge launch).  Below that, about 256 workgroups, a power of two, and no range shorter
    // than 128 keys at full capacity.
    const int pairs = batch * heads;
    if (pairs >= 128) return 1;
    int s = 1;
    while (s * pairs < 256) s *= 2;
    while (s > 1 && capacity / s < 128) s /= 2;
    return s > 64 ? 64 : s;
}

size_t attention_decode_scratch_bytes(int batch, int heads, int d, int splits) {
    if (splits <= 1) return 0;
    return (size_t)batch * heads * splits * (d + 2) * sizeof(float);
}

hipError_t launch_attention_decode(const AttnDecodeArgs& a, hipStream_t s) {
    const dim3 grid(a.splits, a.heads, a.batch), block(256);
    if (a.d == 128) hipLaunchKernelGGL(attn_decode<128>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(attn_decode<64>, grid, block, 0, s, a);
    if (a.splits > 1) {
        const int pairs = a.batch * a.heads;
        if (a.d == 128) hipLaunchKernelGGL(attn_decode_combine<128>, dim3((pairs + 1) / 2), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(attn_decode_combine<64>, dim3((pairs + 3) / 4), dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace eet
