// Dense projections y = x W^T + b with fused epilogues (QKV scatter into the K/V cache,
// add-bias+GELU, add-bias+residual with optional row scatter back to the padded layout).
//
// The paper leaves these to library GEMM calls followed by separate bias/activation kernels
// (Section 3.2 notes that fusion stops at the GEMM calls).  Here the epilogue
// runs on the accumulators, so the intermediate never visits HBM.
//
// Kernels:
//   gemm_mfma_dma64  prefill (M = valid tokens of the batch, packed) and decode steps of many sequences: 256x256 tiles
//                    for the large problems, 128x128, 128x64 and 64x64 when there are few; direct global->LDS loads,
//                    v_mfma_f32_16x16x32_f16; bound by the matrix cores.
//   gemm_flat        decode (M <= 16 rows), small layers: one memory round trip, few instructions.
//   gemm_stream      decode, large layers: every weight is read from HBM exactly once per step, so
//                    the kernel is a weight stream; v_mfma_f32_16x16x32_f16 does the 16-row contraction.
//   gemm_skinny      decode, shapes the two above do not take.
// All compute the transposed tile (weights as the MFMA "A" operand) so that each lane ends up
// with 4 consecutive output columns of one row: 8-byte stores, and 8-byte bias/residual loads.
#include <cstdlib>
#include <mutex>
#include <set>
#include <type_traits>
#include <utility>

#include "kernels.hpp"
#include "pipeline.hpp"

namespace eet {

// --------------------------------------------------------------------------------------------
// epilogue on 4 consecutive output columns n..n+3 of row m
// --------------------------------------------------------------------------------------------
// Operands of the epilogue that come from memory; a latency-bound kernel fetches them before its
// main loop so that no dependent round trip is left after the last MFMA.
struct EpiOperands {
    half4v bias, res;
    int pos;            // QKV only: padded row of the token (prefill) or cache slot n_b (decode)
};

template <int EPI>
__device__ __forceinline__ void epilogue_fetch(const GemmArgs& a, int m, int n, EpiOperands& o) {
    o.bias = *reinterpret_cast<const half4v*>(a.bias + n);
    if (EPI == EPI_BIAS_RES) {
        const int64_t rr = a.res_row_map ? (int64_t)a.res_row_map[m] : (int64_t)m;
        o.res = *reinterpret_cast<const half4v*>(a.res + rr * a.N + n);
    }
    if (EPI == EPI_QKV) o.pos = a.tok_row_map ? a.tok_row_map[m] : a.lens[m];
}

template <int EPI>
__device__ __forceinline__ half4v epilogue_apply(const GemmArgs& a, int m, int n, float v0, float v1, float v2, float v3,
                                                 const EpiOperands& e) {   // returns the four values as stored
    v0 += (float)e.bias[0]; v1 += (float)e.bias[1]; v2 += (float)e.bias[2]; v3 += (float)e.bias[3];
    if (EPI == EPI_BIAS_GELU) {
        v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3);
    }
    if (EPI == EPI_BIAS_RES) {
        v0 += (float)e.res[0]; v1 += (float)e.res[1]; v2 += (float)e.res[2]; v3 += (float)e.res[3];
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
                b_ = e.pos / a.S;
                pos = e.pos - b_ * a.S;
                if (a.left_pad) pos -= a.S - a.lens[b_];
            } else {                             // decode: the new token goes to slot n_b
                b_ = m;
                pos = e.pos;
            }
            if (pos < 0 || pos >= a.max_seq) return o;   // device-side lengths advanced past the capacity (replays the host never saw): drop, never write outside the slots
            const int g = c / a.d, dd = c - g * a.d;
            half_t* cache = which == 1 ? a.k_cache : a.v_cache;
            *reinterpret_cast<half4v*>(cache + (((int64_t)b_ * a.heads + g) * a.max_seq + pos) * a.d + dd) = o;
        }
        return o;
    }
    const int64_t orow = a.out_row_map ? (int64_t)a.out_row_map[m] : (int64_t)m;
    *reinterpret_cast<half4v*>(a.y + orow * a.N + n) = o;
    return o;
}

template <int EPI>
__device__ __forceinline__ void epilogue4(const GemmArgs& a, int m, int n, float v0, float v1, float v2, float v3) {
    EpiOperands e;
    epilogue_fetch<EPI>(a, m, n, e);
    epilogue_apply<EPI>(a, m, n, v0, v1, v2, v3, e);
}

// --------------------------------------------------------------------------------------------
// epilogue of the MFMA tile kernels, through LDS
// --------------------------------------------------------------------------------------------
// The accumulator layout gives a lane one row and 4 consecutive columns: stored like that, a wave-level store
// touches 32 rows with 16 bytes each, and the output (as large as an operand) leaves the chip at a fraction of
// the memory rate.  Instead each wave turns its (AM*16) x 64 tile around in a private piece of the operand
// stages, which are free after the main loop: the residual tile comes in with whole-line loads, the epilogue
// arithmetic runs in fp32 on the accumulators, the rounded tile goes out with whole-line stores (8 rows x 128
// bytes per instruction).  Rows are 128 bytes; their sixteen 8-byte units are XOR-permuted by (row/2)%16 so that
// both access patterns spread over all banks.  `stage`: AM*16*128 bytes of LDS no other wave touches; mw, nw:
// first row and column of the wave tile (its 64 columns are inside N or outside as a whole: N % 64 == 0).
// A wave tile of 128 columns (ANT = 8 accumulator blocks across) is turned around in two passes of 64 columns, J0 = 0 and 4.
// Row bookkeeping of a wave tile's whole-line accesses (lane -> row it*8 + lane/8 of the tile, it = 0 .. AM*2-1), looked up
// once for both 64-column passes and with every lookup in flight together: r0 = output row (EPI_QKV: the sequence
// whose cache the row's K and V go to), r1 = residual row (EPI_QKV: the cache slot; negative or >= max_seq: dropped).
// Rows past M repeat row M-1; they are never stored.
template <int AM, int EPI>
__device__ __forceinline__ void epilogue_rows(const GemmArgs& a, int mw, int lane, int (&r0)[AM * 2], int (&r1)[AM * 2]) {
    const int r8 = lane >> 3;
    int m[AM * 2];
#pragma unroll
    for (int it = 0; it < AM * 2; ++it) {
        m[it] = mw + it * 8 + r8;
        m[it] = m[it] < a.M ? m[it] : a.M - 1;
    }
    if constexpr (EPI == EPI_QKV) {
        if (a.tok_row_map) {                             // prefill: token -> (sequence, position)
            int tok[AM * 2];
#pragma unroll
            for (int it = 0; it < AM * 2; ++it) tok[it] = a.tok_row_map[m[it]];
#pragma unroll
            for (int it = 0; it < AM * 2; ++it) {
                r0[it] = tok[it] / a.S;
                r1[it] = tok[it] - r0[it] * a.S;
            }
            if (a.left_pad) {                            // pads lead: token 0 of the sequence is at row S - L_b
                int len[AM * 2];
#pragma unroll
                for (int it = 0; it < AM * 2; ++it) len[it] = a.lens[r0[it]];
#pragma unroll
                for (int it = 0; it < AM * 2; ++it) r1[it] -= a.S - len[it];
            }
        } else {                                         // decode: the new token goes to slot n_b
#pragma unroll
            for (int it = 0; it < AM * 2; ++it) {
                r0[it] = m[it];
                r1[it] = a.lens[m[it]];
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < AM * 2; ++it) {
            r0[it] = a.out_row_map ? a.out_row_map[m[it]] : m[it];
            r1[it] = (EPI == EPI_BIAS_RES && a.res_row_map) ? a.res_row_map[m[it]] : m[it];
        }
    }
}

// The residual rows under 64 columns of a wave tile, as whole lines (16-byte chunk lane%8 of each row): every request is
// issued before anything waits for one, so the tile costs one trip to memory instead of one per group of rows
// (8192 x 16384 x 2048 with a residual: 634 -> 552 us; 25082 x 12288 x 12288: 6.56 -> 6.37 ms).
template <int AM>
__device__ __forceinline__ void epilogue_request_residual(const GemmArgs& a, half8v (&rv)[AM * 2], const int (&rrow)[AM * 2], int nw, int lane) {
    if (nw >= a.N) return;
    const int c8 = lane & 7;
#pragma unroll
    for (int it = 0; it < AM * 2; ++it) rv[it] = *reinterpret_cast<const half8v*>(a.res + (int64_t)rrow[it] * a.N + nw + c8 * 8);
}

template <int AM, int ANT, int J0, int EPI, bool NTS, int RV>
__device__ __forceinline__ void epilogue_via_lds(const GemmArgs& a, const float4v (&acc)[AM][ANT], const half8v (&rv)[RV],
                                                 const int (&r0)[AM * 2], const int (&r1)[AM * 2], char* stage, int mw, int nw, int lane) {
    static_assert(J0 + 4 <= ANT, "64 columns per pass");
    static_assert(EPI != EPI_BIAS_RES || RV == AM * 2, "the residual lines of the pass, from epilogue_request_residual");
    constexpr int AN = 4;
    constexpr int ROWS = AM * 16;                         // rows of the wave tile
    const int M = a.M, N = a.N;
    if (nw >= N) return;
    const int r8 = lane >> 3, c8 = lane & 7;              // whole-line pattern: row it*8 + r8, 16-byte chunk c8
    if constexpr (EPI == EPI_BIAS_RES) {
#pragma unroll
        for (int it = 0; it < ROWS / 8; ++it) {
            const int row = it * 8 + r8;
            half8v v = rv[it];
            const int sw = (row >> 1) & 15;
            if (sw & 1) v = __builtin_shufflevector(v, v, 4, 5, 6, 7, 0, 1, 2, 3);
            *reinterpret_cast<half8v*>(stage + row * 128 + ((c8 ^ (sw >> 1)) * 16)) = v;
        }
    }
    // arithmetic on the accumulators: acc[i][j][0..3] = row i*16 + lane%16, columns j*16 + (lane/16)*4 ..+4
#pragma unroll
    for (int j = 0; j < AN; ++j) {
        const int unit = j * 4 + (lane >> 4);             // 8-byte unit of the 128-byte row
        const half4v bias = *reinterpret_cast<const half4v*>(a.bias + nw + unit * 4);
#pragma unroll
        for (int i = 0; i < AM; ++i) {
            const int row = i * 16 + (lane & 15);
            half4v* slot = reinterpret_cast<half4v*>(stage + row * 128 + ((unit ^ ((row >> 1) & 15)) * 8));
            float v0 = acc[i][J0 + j][0] + (float)bias[0], v1 = acc[i][J0 + j][1] + (float)bias[1];
            float v2 = acc[i][J0 + j][2] + (float)bias[2], v3 = acc[i][J0 + j][3] + (float)bias[3];
            if (EPI == EPI_BIAS_GELU) {
                v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3);
            }
            if (EPI == EPI_BIAS_RES) {
                const half4v r = *slot;
                v0 += (float)r[0]; v1 += (float)r[1]; v2 += (float)r[2]; v3 += (float)r[3];
            }
            *slot = half4v{(half_t)v0, (half_t)v1, (half_t)v2, (half_t)v3};
        }
    }
    // whole lines out
#pragma unroll
    for (int it = 0; it < ROWS / 8; ++it) {
        const int row = it * 8 + r8, m = mw + row;
        if (m >= M) continue;
        const int sw = (row >> 1) & 15;
        half8v v = *reinterpret_cast<const half8v*>(stage + row * 128 + ((c8 ^ (sw >> 1)) * 16));
        if (sw & 1) v = __builtin_shufflevector(v, v, 4, 5, 6, 7, 0, 1, 2, 3);
        const int n = nw + c8 * 8;
        half_t* dst;
        if (EPI == EPI_QKV) {
            const int which = n / a.hidden;              // 0 = Q, 1 = K, 2 = V
            const int c = n - which * a.hidden;
            if (which == 0) {
                dst = a.y + (int64_t)m * a.hidden + c;
            } else {
                const int b_ = r0[it], pos = r1[it];
                if (pos < 0 || pos >= a.max_seq) continue;   // see epilogue_apply: never outside the sequence's slots
                const int g = c / a.d, dd = c - g * a.d;
                dst = (which == 1 ? a.k_cache : a.v_cache) + (((int64_t)b_ * a.heads + g) * a.max_seq + pos) * a.d + dd;
            }
        } else {
            dst = a.y + (int64_t)r0[it] * (a.ldy ? a.ldy : N) + n;
        }
        if constexpr (NTS) __builtin_nontemporal_store(v, reinterpret_cast<half8v*>(dst));   // an output too large to stay cached for its reader
        else *reinterpret_cast<half8v*>(dst) = v;
    }
}

// --------------------------------------------------------------------------------------------
// MFMA tile kernel
// --------------------------------------------------------------------------------------------
// Tile order: pipe::tile_of_block (pipeline.hpp; the host-side audit checks that it visits every tile exactly once).
// --------------------------------------------------------------------------------------------
// MFMA tile kernel with direct global->LDS loads
// --------------------------------------------------------------------------------------------
// BM x BN tile (256x256 for the large problems, 128x128 and 128x64 for fewer tiles), WGM x WGN waves with wave tiles
// of 64 columns, K steps of 64 through NS LDS stages filled by
// global_load_lds_dwordx4 (no staging registers, no ds_write): with two stages the loads of K step kt+1 are issued
// at the start of step kt, with three (the small tiles, where few workgroups share a CU and nothing else hides the
// trip to memory) those of step kt+2.  An LDS row is the 128 bytes of one operand row, and a wave-level load
// covers 8 rows x 128 bytes, i.e. whole cache lines.  Instead of padding, the eight 16-byte chunks
// of a row are XOR-permuted by (row/2)%8 -- applied on the global address of each lane when loading
// and on the LDS address when reading fragments -- which spreads consecutive rows over all banks.
// MFMA fragments are double-buffered in registers: the reads of the next quarter-step are issued
// before the MFMAs of the current one.
//
// Fragment reads and every wait in the main loop are inline assembly / raw builtins.  The compiler
// cannot tell that an LDS read does not alias an in-flight global->LDS load and would otherwise
// drain all of them (vmcnt(0)) before each read and before each barrier, which undoes the pipeline.

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds + 16*l (the LDS
// base must be wave-uniform).  Kept out of the templates: the builtin only exists for the device.
__device__ __forceinline__ void load_lds_16B(const half_t* gptr, half_t* lds) {
    __builtin_amdgcn_global_load_lds(gptr, lds, 16, 0, 0);
}

template <int N>
__device__ __forceinline__ void wait_lgkm() {
    static_assert(N == 0 || N == 3 || N == 4 || N == 6 || N == 8, "add the count");
    if (N == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (N == 3) asm volatile("s_waitcnt lgkmcnt(3)" ::: "memory");
    if (N == 4) asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");
    if (N == 6) asm volatile("s_waitcnt lgkmcnt(6)" ::: "memory");
    if (N == 8) asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    static_assert(N == 0 || N == 6 || N == 8 || N == 16, "add the count");
    if (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    if (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    if (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
}

// The instructions of the tile kernel's K loop.  The loop itself -- which stage is loaded, read, waited for and released
// when -- is pipe::gemm_k_loop (pipeline.hpp), shared with the host-side audit of the hand-over; this executor supplies the
// instructions, all forced inline.  (Namespace scope because a local class cannot have member templates.)
//
// Matrix instruction: v_mfma_f32_16x16x32_f16.  Under this part's power management the 16x16x32 form sustains about a
// sixth more than 32x32x16 (measured with bare loops of either: 2.08 against 1.79 PFLOP/s over tens of milliseconds): per
// flop it reads and writes half the accumulator registers.  Weights are the A operand (16 output columns x 32 k), the
// activations the B operand (32 k x 16 rows): a lane holds 4 consecutive output columns of one row.
// A wave tile of WM x WN is AM = WM/16 by AN = WN/16 accumulator blocks (WN = 64, or 128 for the four-wave 256 x 256 tile,
// whose 64 blocks per wave live in the accumulation registers).  With two waves per SIMD (pipe::gemm_k_loop) a K tile of
// 64 is walked in four sub-steps s = 2h + mh: k half h (32 columns) times row half mh (AM/2 blocks).  The weight
// fragments of a k half (AN reads of 16 bytes per lane) serve both row halves and are read with the first; every sub-step
// reads AM/2 activation fragments; both kinds are double-buffered in registers, so the reads of sub-step s+1 fly during
// the AM/2 * AN multiplies of sub-step s, and the other wave of the SIMD covers what still shows.  With one wave per SIMD
// (pipe::gemm_k_loop_interleaved) nothing covers a stall, and a burst of LDS reads stalls the issuing wave, multiplies
// included, until the LDS queue drains (16 reads in a row in front of 64 multiplies: 1840 cycles against 1055 for the
// multiplies alone; one read after every third multiply: 1080); there the fragments of a whole k half are
// double-buffered and every request sits between two multiplies.
template <int BM, int BN, int NW, int NS, int KS, int AM, int AN>
struct GemmTileExec {
    static constexpr int BK = 64, AH = AM / 2;
    static constexpr int LRA = BM / NW, LRW = BN / NW, LIA = LRA / 8, LIW = LRW / 8;
    static_assert(AM % 2 == 0 && AH >= 1 && AH <= 4 && (AN == 4 || AN == 8), "wave tile shape");
    const half_t* pa[LIA];                 // this lane's source of each load instruction, K tile 0
    const half_t* pw[LIW];
    half_t* as_base;                       // stage 0 of this wave's K group: As[kg * NS], Ws[kg * NS]
    half_t* ws_base;
    unsigned a_lds, w_lds;                 // LDS byte address of row lane%16 of the wave tile's first block, stage 0
    unsigned foff[2];                      // byte offset of this lane's 16 bytes of k half h inside the (permuted) row
    int kg, wave;
    half8v fa[2][AH], fw[2][AN];           // fa[s & 1]: activations of sub-step s; fw[h & 1]: weights of k half h
    half8v ga[2][AM], gw[2][AN];           // the one-wave-per-SIMD schedule: all fragments of k half h
    float4v acc[AM][AN];

    __device__ __forceinline__ void load(int tile, int stage) {
#pragma unroll
        for (int v = 0; v < LIA; ++v)
            load_lds_16B(pa[v] + (int64_t)(tile * KS + kg) * BK, as_base + stage * (BM * BK) + (wave * LRA + v * 8) * BK);
#pragma unroll
        for (int v = 0; v < LIW; ++v)
            load_lds_16B(pw[v] + (int64_t)(tile * KS + kg) * BK, ws_base + stage * (BN * BK) + (wave * LRW + v * 8) * BK);
    }
    template <int L>
    __device__ __forceinline__ void wait_vmem() {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L * (LIA + LIW)) : "memory");
    }
    __device__ __forceinline__ void barrier() { __builtin_amdgcn_s_barrier(); }
    // LDS reads of sub-step SUB: 16 bytes per lane per fragment, blocks 2 KB apart
    static constexpr int reads_of(int sub) { return AH + ((sub & 1) == 0 ? AN : 0); }
#define EET_DREAD(DST, ADDR, OFF) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(DST) : "v"(ADDR), "n"(OFF) : "memory")
    template <int BUF, int SUB>
    __device__ __forceinline__ void frag(int stage) {
        static_assert(BUF == (SUB & 1), "activation buffer of a sub-step");
        constexpr int H = SUB >> 1, MH = SUB & 1;
        const unsigned va_ = a_lds + stage * (BM * BK * 2) + foff[H];
        EET_DREAD(fa[BUF][0], va_, (MH * AH + 0) * 2048);
        if (AH > 1) EET_DREAD(fa[BUF][1 % AH], va_, (MH * AH + 1) * 2048);
        if (AH > 2) EET_DREAD(fa[BUF][2 % AH], va_, (MH * AH + 2) * 2048);
        if (AH > 3) EET_DREAD(fa[BUF][3 % AH], va_, (MH * AH + 3) * 2048);
        if (MH == 0) {
            const unsigned vw_ = w_lds + stage * (BN * BK * 2) + foff[H];
            EET_DREAD(fw[H][0], vw_, 0);
            EET_DREAD(fw[H][1], vw_, 2048);
            EET_DREAD(fw[H][2], vw_, 4096);
            EET_DREAD(fw[H][3], vw_, 6144);
            if (AN > 4) {
                EET_DREAD(fw[H][4 % AN], vw_, 8192);
                EET_DREAD(fw[H][5 % AN], vw_, 10240);
                EET_DREAD(fw[H][6 % AN], vw_, 12288);
                EET_DREAD(fw[H][7 % AN], vw_, 14336);
            }
        }
    }
#undef EET_DREAD
    // The reads of sub-step SUB have landed; those of sub-step NEWER (issued after them; -1: none) may stay in flight.
    template <int BUF, int SUB, int NEWER>
    __device__ __forceinline__ void wait_frag() {
        static_assert(BUF == (SUB & 1), "activation buffer of a sub-step");
        asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(NEWER < 0 ? 0 : reads_of(NEWER & 3)) : "memory");
#pragma unroll
        for (int i = 0; i < AH; ++i) asm volatile("" : "+v"(fa[BUF][i]));      // the fragments are defined from here on
        if ((SUB & 1) == 0) {
#pragma unroll
            for (int j = 0; j < AN; ++j) asm volatile("" : "+v"(fw[SUB >> 1][j]));
        }
    }
    // ---- the one-wave-per-SIMD schedule (pipe::gemm_k_loop_interleaved): whole k halves, double-buffered -------------
    // LDS read number R of k half H into buffer H: the AN weight fragments, then the AM activation fragments
    template <int H, int R>
    __device__ __forceinline__ void half_read(unsigned va_, unsigned vw_) {
        if constexpr (R < AN) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(gw[H][R % AN]) : "v"(vw_), "n"(R * 2048) : "memory");
        else asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(ga[H][(R - AN) % AM]) : "v"(va_), "n"((R - AN) * 2048) : "memory");
    }
    template <int H, int... R>
    __device__ __forceinline__ void half_read_all(unsigned va_, unsigned vw_, std::integer_sequence<int, R...>) {
        (half_read<H, R>(va_, vw_), ...);
    }
    template <int H>
    __device__ __forceinline__ void fetch_half(int stage) {
        half_read_all<H>(a_lds + stage * (BM * BK * 2) + foff[H], w_lds + stage * (BN * BK * 2) + foff[H], std::make_integer_sequence<int, AM + AN>{});
    }
    __device__ __forceinline__ void wait_fetched() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int j = 0; j < AN; ++j) asm volatile("" : "+v"(gw[h][j]));
#pragma unroll
            for (int i = 0; i < AM; ++i) asm volatile("" : "+v"(ga[h][i]));
        }
    }
    // multiply number IDX of k half H, followed by its share of the side work: the reads of the other k half and the tile
    // loads, each spread over the first three quarters of the phase (the last quarter lets the reads land; loads issued
    // later arrive later); scheduling barriers pin each request between the two multiplies it was written between
    template <int H, bool LOAD, int IDX>
    __device__ __forceinline__ void half_mma_one(unsigned va_, unsigned vw_, int64_t koff, int lstage) {
        constexpr int MF = AM * AN, NR = AM + AN, NL = LIA + LIW;
        constexpr int RS = (MF * 3 / 4) / NR, LS = (MF * 3 / 4) / NL;   // multiplies per read, per load (both measured best at 3 for 64)
        static_assert(RS >= 1 && LS >= 1, "side work fits between the multiplies");
        constexpr int i = IDX / AN, j = IDX % AN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(gw[H][j], ga[H][i], acc[i][j], 0, 0, 0);
        if constexpr (IDX % RS == 0 && IDX / RS < NR) {
            __builtin_amdgcn_sched_barrier(0);
            half_read<1 - H, IDX / RS>(va_, vw_);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (LOAD && IDX % LS == LS / 2 && IDX / LS < NL) {
            constexpr int v = IDX / LS;
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (v < LIA) load_lds_16B(pa[v % LIA] + koff, as_base + lstage * (BM * BK) + (wave * LRA + v * 8) * BK);
            else load_lds_16B(pw[(v - LIA) % LIW] + koff, ws_base + lstage * (BN * BK) + (wave * LRW + (v - LIA) * 8) * BK);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    template <int H, bool LOAD, int... I>
    __device__ __forceinline__ void half_mma_seq(unsigned va_, unsigned vw_, int64_t koff, int lstage, std::integer_sequence<int, I...>) {
        __builtin_amdgcn_sched_barrier(0);
        (half_mma_one<H, LOAD, I>(va_, vw_, koff, lstage), ...);
        __builtin_amdgcn_sched_barrier(0);
    }
    template <int H>
    __device__ __forceinline__ void mma_half_fetch(int stage) {
        half_mma_seq<H, false>(a_lds + stage * (BM * BK * 2) + foff[1 - H], w_lds + stage * (BN * BK * 2) + foff[1 - H], 0, 0,
                               std::make_integer_sequence<int, AM * AN>{});
    }
    template <int H>
    __device__ __forceinline__ void mma_half_fetch_load(int stage, int tile, int lstage) {
        half_mma_seq<H, true>(a_lds + stage * (BM * BK * 2) + foff[1 - H], w_lds + stage * (BN * BK * 2) + foff[1 - H],
                              (int64_t)(tile * KS + kg) * BK, lstage, std::make_integer_sequence<int, AM * AN>{});
    }
    template <int BUF, int SUB>
    __device__ __forceinline__ void mma() {
        static_assert(BUF == (SUB & 1), "activation buffer of a sub-step");
        constexpr int H = SUB >> 1, MH = SUB & 1;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < AH; ++i)
#pragma unroll
            for (int j = 0; j < AN; ++j)
                acc[MH * AH + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[H][j], fa[BUF][i], acc[MH * AH + i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
};

// SCHED: 0 = the schedule of pipe::gemm_k_loop<NS>, 1 = its early-release form (two stages), 2 = the schedule for one wave
// per SIMD (pipe::gemm_k_loop_interleaved; two stages, one K group)
// NTS: the output is stored with the non-temporal hint (outputs of 256 MB and more, which no cache keeps for their reader:
// 24576 x 49152 x 12288 21.70 -> 21.53 ms, 24576 x 12288 x 12288 5.69 -> 5.59, 8192 x 16384 x 12288 2.436 -> 2.393).
template <int BM, int BN, int WGM, int WGN, int EPI, int NS, int KS, int SCHED, bool NTS = false>
__global__ __launch_bounds__(WGM* WGN* KS * 64) void gemm_mfma_dma64(GemmArgs a, int tiles_m, int tiles_n) {
    static_assert(SCHED == 0 || (NS == 2 && KS == 1 && (SCHED == 1 || SCHED == 2)), "schedule");
    // KS > 1: KS groups of WGM x WGN waves share the tile and take every KS-th K step each, through LDS stages of their
    // own; the other groups' accumulators are added to the first's through LDS at the end.  For the few
    // tiles of a narrow output with a long K, where nothing else puts more loads in flight per CU.
    constexpr int NW = WGM * WGN, BK = 64;
    static_assert(NS == 2 || NS == 3, "LDS stages");
    static_assert(KS == 1 || KS == 2, "K groups");
    constexpr int WM = BM / WGM, WN = BN / WGN, AM = WM / 16, AN = WN / 16;   // wave tile in 16 x 16 accumulator blocks
    constexpr int LRA = BM / NW, LRW = BN / NW;   // rows of each operand tile a wave loads per K step
    constexpr int LIA = LRA / 8, LIW = LRW / 8;   // wave-level load instructions per operand per K step
    static_assert(LRA % 8 == 0 && LRW % 8 == 0 && LIA >= 1 && LIW >= 1 && WM % 32 == 0 && (WN == 64 || WN == 128), "tile shape");
    __shared__ __attribute__((aligned(1024))) half_t As[KS * NS][BM * BK];
    __shared__ __attribute__((aligned(1024))) half_t Ws[KS * NS][BN * BK];

    int tile_m, tile_n;
    pipe::tile_of_block((int)blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction: keeps LDS bases in scalar registers
    const int kg = KS == 1 ? 0 : wv / NW;                    // K group of this wave
    const int wave = KS == 1 ? wv : wv % NW;                 // wave inside its group
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    const int M = a.M, N = a.N, K = a.K;
    const int nk = K / (BK * KS);                            // steps of this group (the host sends whole multiples)

    GemmTileExec<BM, BN, NW, NS, KS, AM, AN> ex;
    static_assert(decltype(ex)::LIA == LIA && decltype(ex)::LIW == LIW, "load instructions per K step");
    ex.kg = kg;
    ex.wave = wave;
    ex.as_base = &As[kg * NS][0];
    ex.ws_base = &Ws[kg * NS][0];
#pragma unroll
    for (int v = 0; v < LIA; ++v) {
        const int row = wave * LRA + v * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        int gr = m0 + row;
        gr = gr < M ? gr : M - 1;
        ex.pa[v] = a.x + (int64_t)gr * (a.lda ? a.lda : K) + c * 8;
    }
#pragma unroll
    for (int v = 0; v < LIW; ++v) {
        const int row = wave * LRW + v * 8 + (lane >> 3);
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        int gr = n0 + row;
        gr = gr < N ? gr : N - 1;
        ex.pw[v] = a.w + (int64_t)gr * K + c * 8;
    }
    // fragment rows: lane l reads row l%16 of a block, the 16 bytes (l/16) of k half h; rows are 128 bytes with their
    // 16-byte chunks XOR-permuted by (row/2)%8, and blocks start at multiples of 16 rows, so the permutation is the lane's own
    const int frow = lane & 15, fG = lane >> 4, fsw = frow >> 1;
    ex.a_lds = (unsigned)(uintptr_t)&As[kg * NS][(wm0 + frow) * BK];
    ex.w_lds = (unsigned)(uintptr_t)&Ws[kg * NS][(wn0 + frow) * BK];
#pragma unroll
    for (int h = 0; h < 2; ++h) ex.foff[h] = (unsigned)(((h * 4 + fG) ^ fsw) * 16);

    float4v (&acc)[AM][AN] = ex.acc;
#pragma unroll
    for (int i = 0; i < AM; ++i)
#pragma unroll
        for (int j = 0; j < AN; ++j) acc[i][j] = float4v{0.f, 0.f, 0.f, 0.f};
    if constexpr (SCHED == 2) pipe::gemm_k_loop_interleaved(ex, nk);
    else pipe::gemm_k_loop<NS, SCHED == 1>(ex, nk);

    __syncthreads();                                      // every wave is done with the operand stages
    if constexpr (KS > 1) {
        // the other groups' partial tiles go over the weight stages, lane-major (no bank conflicts), to the first
        constexpr int PT = AM * AN * 4 * 64;                  // floats of one wave's partial tile
        static_assert((KS - 1) * NW * PT * 4 <= (int)sizeof(Ws), "partial tiles over the weight stages");
        float* red = reinterpret_cast<float*>(&Ws[0][0]) + wave * PT + lane;
        if (kg > 0) {
            float* mine = red + (kg - 1) * (NW * PT);
#pragma unroll
            for (int i = 0; i < AM; ++i)
#pragma unroll
                for (int j = 0; j < AN; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mine[((i * AN + j) * 4 + r) * 64] = acc[i][j][r];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int g = 0; g < KS - 1; ++g)
#pragma unroll
            for (int i = 0; i < AM; ++i)
#pragma unroll
                for (int j = 0; j < AN; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[i][j][r] += red[g * (NW * PT) + ((i * AN + j) * 4 + r) * 64];
    }
    constexpr int EB = WM * 128;                           // bytes of a wave's turn-around area
    // row lookups and residual lines of the wave tile: all requested here, consumed by the passes below
    int er0[AM * 2], er1[AM * 2];
    epilogue_rows<AM, EPI>(a, m0 + wm0, lane, er0, er1);
    constexpr int RV = EPI == EPI_BIAS_RES ? AM * 2 : 1;
    half8v rv0[RV], rv1[AN == 8 ? RV : 1];
    if constexpr (EPI == EPI_BIAS_RES) {
        epilogue_request_residual<AM>(a, rv0, er1, n0 + wn0, lane);
        if constexpr (AN == 8) epilogue_request_residual<AM>(a, rv1, er1, n0 + wn0 + 64, lane);
    }
    // with K groups the partial tiles above sit in the weight stages and group 0 may still be summing them while a faster
    // wave of the group already turns its tile around: that must then happen in the activation stages only
    static_assert(KS == 1 || NW * EB <= (int)sizeof(As), "turn-around areas must not touch the partial tiles");
    if constexpr (NW * EB <= (int)sizeof(As)) {
        char* area = reinterpret_cast<char*>(&As[0][0]) + wave * EB;
        epilogue_via_lds<AM, AN, 0, EPI, NTS>(a, acc, rv0, er0, er1, area, m0 + wm0, n0 + wn0, lane);
        if constexpr (AN == 8) epilogue_via_lds<AM, AN, 4, EPI, NTS>(a, acc, rv1, er0, er1, area, m0 + wm0, n0 + wn0 + 64, lane);   // second 64 columns, same area
    } else {
        static_assert(NW == 8 && AN == 4 && 4 * EB <= (int)sizeof(As) && 4 * EB <= (int)sizeof(Ws), "turn-around areas");
        epilogue_via_lds<AM, AN, 0, EPI, NTS>(a, acc, rv0, er0, er1, reinterpret_cast<char*>(wave < 4 ? &As[0][0] : &Ws[0][0]) + (wave & 3) * EB,
                                         m0 + wm0, n0 + wn0, lane);
    }
}

// --------------------------------------------------------------------------------------------
// weight-streaming kernel for M <= 16 rows per grid.y slice
// --------------------------------------------------------------------------------------------
// Workgroup = NW waves; it owns 16*NF output columns.  K steps of 32 are dealt round-robin to
// the waves (adjacent waves read adjacent 64-byte pieces of the same weight rows).
// LN = true fuses the LayerNorm that precedes the projection (decode: LN1 -> QKV, LN2 -> FFN-1):
// every workgroup first computes mean and 1/std of its <= 16 activation rows (two passes over
// rows that stay in L1/L2), then normalises the activation fragments on their way into the MFMA,
// so the normalised activations never exist in memory and one launch per projection is saved.
// BUMP: the workgroup with blockIdx 0 also advances the per-sequence cache lengths (n_b += 1).
template <int NF, int EPI, bool LN, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_skinny(GemmArgs a) {
    constexpr int UN = 4;                       // K steps in flight per wave
    __shared__ float red[NW][NF * 16][17];
    __shared__ float ln_mean[16], ln_rstd[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, G = lane >> 4;
    const int n0 = blockIdx.x * (NF * 16), mc = blockIdx.y * 16;
    const int M = a.M, N = a.N, K = a.K;
    const int nsteps = K / 32;

    if (a.bump_lens != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && tid < a.bump_count) a.bump_lens[tid] += 1;

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

    // The weight (and gamma/beta) fragments of a chunk of UN K steps are requested one chunk ahead
    // of their use; the first chunk is requested before the LayerNorm statistics, whose latency
    // (two passes over cached activation rows) then hides behind the first trip to HBM.
    half8v xf[UN], wf[UN][NF], gf[UN], bf[UN];
    auto request = [&](int s0) {
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int step = s0 + NW * u;
            const int k = (step < nsteps ? step : wave) * 32;      // past the end: any valid step, zeroed below
            xf[u] = *reinterpret_cast<const half8v*>(xp + k);
            if (LN) {
                gf[u] = *reinterpret_cast<const half8v*>(a.ln_gamma + k + G * 8);
                bf[u] = *reinterpret_cast<const half8v*>(a.ln_beta + k + G * 8);
            }
#pragma unroll
            for (int f = 0; f < NF; ++f) wf[u][f] = *reinterpret_cast<const half8v*>(wp[f] + k);
        }
    };
    if (wave < nsteps) request(wave);
    float mean = 0.f, rstd = 1.f;
    if (LN) {
        // 16 threads per row: thread (row = tid/16, sub = tid%16) walks the row in 16-byte vectors
        const int row = (tid >> 4) & 15, sub = tid & 15;       // (workgroups wider than 256 threads repeat the work)
        int rr = mc + row;
        rr = rr < M ? rr : M - 1;
        const half_t* rp = a.x + (int64_t)rr * K;
        // loads go out in batches of 8 independent 16-byte vectors (a scalar loop would pay one
        // memory round trip per vector)
        float sum = 0.f;
        for (int c0 = sub * 8; c0 < K; c0 += 8 * 128) {
            half8v v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int cidx = c0 + i * 128;
                v[i] = *reinterpret_cast<const half8v*>(rp + (cidx < K ? cidx : sub * 8));
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (c0 + i * 128 < K) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) sum += (float)v[i][e];
                }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, kWave);
        const float mu = sum / (float)K;
        float sq = 0.f;
        for (int c0 = sub * 8; c0 < K; c0 += 8 * 128) {
            half8v v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int cidx = c0 + i * 128;
                v[i] = *reinterpret_cast<const half8v*>(rp + (cidx < K ? cidx : sub * 8));
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (c0 + i * 128 < K) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float dlt = (float)v[i][e] - mu;
                        sq += dlt * dlt;
                    }
                }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o, kWave);
        if (sub == 0) {
            ln_mean[row] = mu;
            ln_rstd[row] = rsqrtf(sq / (float)K + a.ln_eps);
        }
        __syncthreads();
        mean = ln_mean[fr];
        rstd = ln_rstd[fr];
    }
    for (int s0 = wave; s0 < nsteps; s0 += NW * UN) {
        half8v cx[UN], cw[UN][NF];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            cx[u] = xf[u];
            if (LN) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    cx[u][e] = (half_t)(((float)xf[u][e] - mean) * rstd * (float)gf[u][e] + (float)bf[u][e]);
            }
            if (s0 + NW * u >= nsteps) {
#pragma unroll
                for (int e = 0; e < 8; ++e) cx[u][e] = (half_t)0.f;
            }
#pragma unroll
            for (int f = 0; f < NF; ++f) cw[u][f] = wf[u][f];
        }
        if (s0 + NW * UN < nsteps) request(s0 + NW * UN);            // next chunk in flight during the MFMAs
#pragma unroll
        for (int u = 0; u < UN; ++u)
#pragma unroll
            for (int f = 0; f < NF; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cw[u][f], cx[u], acc[f], 0, 0, 0);
    }
    // acc[f][r]: output column n0 + f*16 + 4G + r, row mc + lane%16
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][f * 16 + 4 * G + r][fr] = acc[f][r];
    __syncthreads();
    for (int t = tid; t < 64 * NF; t += NW * 64) {
        const int ng = t % (4 * NF), ml = t / (4 * NF);
        const int m = mc + ml, n = n0 + ng * 4;
        if (m >= M || n >= N) continue;
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float part = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) part += red[w][ng * 4 + c][ml];
            v[c] = part;
        }
        epilogue4<EPI>(a, m, n, v[0], v[1], v[2], v[3]);
    }
}

// --------------------------------------------------------------------------------------------
// latency-bound variant of the weight-streaming kernel (small layers)
// --------------------------------------------------------------------------------------------
// When one projection moves only a few MB, its time is a chain of memory round trips plus the
// instructions each wave has to issue (a wave64 vector instruction takes 4 cycles: a thousand of
// them are two microseconds), not bytes.  This variant is built for both:
//   * K = 64 * NW * UPW is a compile-time constant (NW waves, UPW units of 64 K values per wave),
//     so address arithmetic folds into immediate offsets and nothing is conditional;
//   * a workgroup owns TN = 16 output columns (8 when 16 would leave most CUs without work: the
//     staging rows 8..15 then hold nothing and their results are dropped); every wave requests its whole share of the weights at
//     once, after the activation rows and before the epilogue's bias / residual / cache slot:
//     one round trip to memory in all;
//   * every load instruction reads whole 128-byte lines (8 lanes x 16 bytes per row; measured on
//     this part: an instruction that takes 64 bytes from each of 16 lines, which is what the MFMA
//     operand layout asks for, moves data several times slower out of L2).  The MFMA layout is
//     produced in LDS instead: a wave writes each 16 x 128-byte unit it loaded into a private
//     staging area and reads back 16 bytes per lane at (row lane%16, chunk lane/16 + 4u) for the
//     two MFMAs u of the unit.  LDS operations of one wave execute in order, so the private
//     areas need no barrier (and the wave's partial sums reuse the first one);
//   * the activation rows (8, or 16 when M > 8; rows past M repeat row M-1 and their results
//     are never written) are read as contiguous 16-byte vectors spread over all threads and
//     shared through LDS: one barrier, after which every operand fragment is a 16-byte LDS read.
//     With LN a row belongs to 8*NW lanes of one wave: its statistics are reduced by lane
//     exchanges over values held in registers, and the row reaches LDS normalised.
//
// Dynamic LDS: [8 or 16][K + 8] activations, then per wave SA staging areas of 16 x 144 bytes.
constexpr int kFlatStageRow = 72;                           // halves per staged row: 128 bytes + 16 padding
__host__ __device__ constexpr int flat_stage_areas(int nw, int upw) { return (nw >= 16 && upw > 2) ? 2 : upw; }
__host__ __device__ constexpr int flat_lds_bytes(int nw, int upw, int xrows) {
    return xrows * (64 * nw * upw + 8) * 2 + nw * flat_stage_areas(nw, upw) * 16 * kFlatStageRow * 2;
}

// sum over aligned groups of W lanes (W = 32 or 64), result in every lane of the group
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    auto dpp_add = [](float x, auto ctrl) {
        constexpr int c = decltype(ctrl)::value;
        const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), c, 0xf, 0xf, false);
        return x + __builtin_bit_cast(float, y);
    };
    v = dpp_add(v, std::integral_constant<int, 0xb1>{});    // quad_perm [1,0,3,2]: lane ^ 1
    v = dpp_add(v, std::integral_constant<int, 0x4e>{});    // quad_perm [2,3,0,1]: lane ^ 2
    v = dpp_add(v, std::integral_constant<int, 0x141>{});   // row_half_mirror: the other quad of 8
    v = dpp_add(v, std::integral_constant<int, 0x140>{});   // row_mirror: the other half of 16
    v += __shfl_xor(v, 16, kWave);
    if (W == 64) v += __shfl_xor(v, 32, kWave);
    return v;
}

// A launch of the weight-streaming kernels with gridDim.y > 1 (template flag SL) cuts the rows into slices of 16: the
// workgroups of row blockIdx.y see rows [16 y, 16 y + 16) as a problem of their own (a decode step of 17 to 64
// sequences: the slices run side by side and all but the first find the weights in L2).  Used without row maps, fused
// LayerNorm, prefetch workgroups or length bump.  A flag of its own because even this much scalar arithmetic shows in
// the launch-bound decode of small layers (0.2 % of the 24-layer pass).
template <int EPI>
__device__ __forceinline__ void take_row_slice(GemmArgs& a) {
    const int m0 = (int)blockIdx.y * 16;
    const int rows = a.M - m0;
    a.M = rows < 16 ? rows : 16;
    a.x += (size_t)m0 * a.K;
    if (EPI == EPI_QKV) {                       // decode: row m is sequence m, its token goes to slot lens[m] of its own cache
        a.y += (size_t)m0 * a.hidden;
        a.lens += m0;
        const size_t seq = (size_t)a.heads * a.max_seq * a.d;
        a.k_cache += (size_t)m0 * seq;
        a.v_cache += (size_t)m0 * seq;
    } else {
        a.y += (size_t)m0 * a.N;
        if (EPI == EPI_BIAS_RES) a.res += (size_t)m0 * a.N;
    }
}

template <int NW, int UPW, int TN, int EPI, bool LN, bool SL, bool XM = false>
__global__ __launch_bounds__(NW * 64) void gemm_flat(GemmArgs a) {
    static_assert(!XM || (EPI == EPI_BIAS_RES && !LN && !SL), "merging attention ranges: the output projection of a decode step");
    if (SL) take_row_slice<EPI>(a);
    constexpr int NT = NW * 64;
    constexpr int K = 64 * NW * UPW, KV = K / 8, LDX = K + 8;   // LDX: 16-byte reads of 16 rows spread over all banks
    constexpr int SA = flat_stage_areas(NW, UPW);
    constexpr int TPR = NT / 8;                             // LN: lanes per activation row (32 or 64)
    static_assert(!LN || TPR <= 64, "a row's statistics are reduced inside one wave");
    extern __shared__ __attribute__((aligned(16))) unsigned char flat_smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, G = lane >> 4;
    constexpr int WA = TN / 8;                              // load instructions per unit (8 weight rows each)
    const int n0 = blockIdx.x * TN;
    const int M = a.M;
    const int xrows = M <= 8 ? 8 : 16;
    half_t* xs = reinterpret_cast<half_t*>(flat_smem);
    half_t* wst = xs + xrows * LDX + wave * (SA * 16 * kFlatStageRow);
    float* red = reinterpret_cast<float*>(xs + xrows * LDX);            // after the MFMAs: wave w's tile over its staging areas
    constexpr int RW = SA * 16 * kFlatStageRow / 2;                     // floats between the waves' tiles
    static_assert(RW >= 16 * 20, "partial-sum tile must fit the wave's own staging space");

    if (a.pf.blocks > 0 && (int)blockIdx.x >= a.N / TN) {   // extra workgroups: operands of the launches that follow
        run_prefetch(a.pf, (int)blockIdx.x - a.N / TN, a.pf.blocks, tid, NT);
        return;
    }
    if (a.bump_lens != nullptr && blockIdx.x == 0 && tid < a.bump_count) a.bump_lens[tid] += 1;

    // ---- requests, oldest first: activations, weights, epilogue operands --------------------
    // half h of the activations = rows 8h .. 8h+7; thread -> (row, 16-byte vectors) per half:
    //   LN:  row tid/TPR, vectors tid%TPR + TPR*i      (a row stays inside one wave)
    //   else: vector tid + NT*i of the 8*KV vectors of the half
    half8v xv[2][UPW], gv[LN ? UPW : 1], bv[LN ? UPW : 1];
    uint32_t xdst[UPW];                                       // LDS offset (halves) of vector i inside a half
    auto request_x = [&](int h) {
#pragma unroll
        for (int i = 0; i < UPW; ++i) {
            const int row = LN ? tid / TPR : (tid + NT * i) / KV;
            const int col = LN ? tid % TPR + TPR * i : (tid + NT * i) % KV;
            int src = 8 * h + row;
            src = src < M ? src : M - 1;
            xv[h][i] = *reinterpret_cast<const half8v*>(reinterpret_cast<const char*>(a.x) + (uint32_t)(src * K + col * 8) * 2u);
            xdst[i] = row * LDX + col * 8;
            if (LN && h == 0) {
                gv[i] = *reinterpret_cast<const half8v*>(reinterpret_cast<const char*>(a.ln_gamma) + (uint32_t)col * 16u);
                bv[i] = *reinterpret_cast<const half8v*>(reinterpret_cast<const char*>(a.ln_beta) + (uint32_t)col * 16u);
            }
        }
    };
    if (!XM) {
        request_x(0);
        if (M > 8) request_x(1);
    }
    // weights: per unit, lane l takes 16 bytes (chunk l%8) of rows l/8 and 8 + l/8
    const int wrow = lane >> 3, wchunk = lane & 7;
    half8v wreg[UPW][WA];
    {
        const char* wbase = reinterpret_cast<const char*>(a.w) + (size_t)n0 * K * 2;
        const uint32_t woff = (uint32_t)(wrow * K + wave * (UPW * 64) + wchunk * 8) * 2u;
#pragma unroll
        for (int q = 0; q < UPW; ++q)
#pragma unroll
            for (int h = 0; h < WA; ++h)
                wreg[q][h] = *reinterpret_cast<const half8v*>(wbase + woff + (uint32_t)(h * 8 * K + q * 64) * 2u);
    }
    // epilogue operands of the 4*TN threads that write the 16 x TN outputs (no row maps in decode)
    const int eml = tid / (TN / 4), enl = (tid % (TN / 4)) * 4, en = n0 + enl;
    const bool writer = tid < 4 * TN && eml < M;
    EpiOperands eo;
    if (writer) {
        eo.bias = *reinterpret_cast<const half4v*>(a.bias + en);
        if (EPI == EPI_BIAS_RES) eo.res = *reinterpret_cast<const half4v*>(a.res + (uint32_t)(eml * a.N + en));
        if (EPI == EPI_QKV) eo.pos = a.lens[eml];
    }

    // ---- XM: the activations are the attention output of this step, one partial per key range; merge them ----
    // (what attn_decode_combine does in a launch of its own: common maximum, rescaled sums, one division)
    if constexpr (XM) {
        constexpr int MAXS = NW >= 16 ? 2 : 8;                  // ranges in flight at a time (1024 threads: 128 VGPRs each)
        const int splits = a.x_splits;
        auto merge_x = [&](int h) {
#pragma unroll
            for (int i = 0; i < UPW; ++i) {
                const int row = (tid + NT * i) / KV, col = (tid + NT * i) % KV;
                const int src = 8 * h + row;
                xdst[i] = row * LDX + col * 8;
                half8v o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (half_t)0.f;
                if (src < M) {                                  // rows past M feed outputs nobody writes
                    const int g = (col * 8) / a.d, dd = (col * 8) % a.d;
                    const int64_t bh = (int64_t)src * a.heads + g;
                    const float* ml = a.x_part_ml + bh * splits * 2;
                    const float* pa = a.x_part_acc + bh * splits * a.d + dd;
                    float lsum = 0.f, av[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) av[e] = 0.f;
                    auto fetch = [&](int s0, float2v (&mlv)[MAXS], float4v (&lo)[MAXS], float4v (&hi)[MAXS]) {
#pragma unroll
                        for (int u = 0; u < MAXS; ++u) {
                            const int s = s0 + u < splits ? s0 + u : splits - 1;
                            mlv[u] = *reinterpret_cast<const float2v*>(ml + s * 2);
                            lo[u] = *reinterpret_cast<const float4v*>(pa + (int64_t)s * a.d);
                            hi[u] = *reinterpret_cast<const float4v*>(pa + (int64_t)s * a.d + 4);
                        }
                    };
                    auto add = [&](int s0, float mx, const float2v (&mlv)[MAXS], const float4v (&lo)[MAXS], const float4v (&hi)[MAXS]) {
#pragma unroll
                        for (int u = 0; u < MAXS; ++u) {
                            const float sc = s0 + u < splits ? exp2f(mlv[u][0] - mx) : 0.f;
                            lsum += mlv[u][1] * sc;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                av[e] += lo[u][e] * sc;
                                av[4 + e] += hi[u][e] * sc;
                            }
                        }
                    };
                    float2v mlv[MAXS];
                    float4v lo[MAXS], hi[MAXS];
                    if (splits <= MAXS) {                       // the usual case: everything in one trip to memory
                        fetch(0, mlv, lo, hi);
                        float mx = mlv[0][0];                   // empty ranges report a finite maximum and a zero sum (clamped slots repeat the last range)
#pragma unroll
                        for (int u = 1; u < MAXS; ++u) mx = fmaxf(mx, mlv[u][0]);
                        add(0, mx, mlv, lo, hi);
                    } else {
                        float mx = -INFINITY;
                        for (int s = 0; s < splits; ++s) mx = fmaxf(mx, ml[s * 2]);
                        for (int s0 = 0; s0 < splits; s0 += MAXS) {
                            fetch(s0, mlv, lo, hi);
                            add(s0, mx, mlv, lo, hi);
                        }
                    }
                    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;     // a pair that saw no key at all: zeros, not 0/0
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = (half_t)(av[e] * inv);
                }
                xv[h][i] = o;
            }
        };
        merge_x(0);
        if (M > 8) merge_x(1);
    }

    // ---- activations -> LDS (normalised when LN) ----------------------------------------------
    auto publish_x = [&](int h) {
        if (LN) {
            // shifted sums: d = x - p with p the row's first element keeps the variance formula
            // free of cancellation whatever the row's mean is
            const half_t p = (half_t)__shfl((float)xv[h][0][0], lane & ~(TPR - 1), kWave);
            const half2v p2 = {p, p}, one2 = {(half_t)1.f, (half_t)1.f};
            float sd = 0.f, sq = 0.f;
#pragma unroll
            for (int i = 0; i < UPW; ++i)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const half2v d2 = half2v{xv[h][i][e], xv[h][i][e + 1]} - p2;
                    sd = __builtin_amdgcn_fdot2(d2, one2, sd, false);
                    sq = __builtin_amdgcn_fdot2(d2, d2, sq, false);
                }
            sd = group_sum<TPR>(sd);
            sq = group_sum<TPR>(sq);
            const float md = sd * (1.0f / K);
            const float mu = (float)p + md;
            const float rstd = rsqrtf(fmaxf(sq * (1.0f / K) - md * md, 0.f) + a.ln_eps);
#pragma unroll
            for (int i = 0; i < UPW; ++i) {
                half8v o;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // three fused multiply-adds that take their fp16 operand directly
                    const float sc = __builtin_fmaf((float)gv[i][e], rstd, 0.f);
                    const float sh = __builtin_fmaf(-mu, sc, (float)bv[i][e]);
                    o[e] = (half_t)__builtin_fmaf((float)xv[h][i][e], sc, sh);
                }
                *reinterpret_cast<half8v*>(&xs[8 * h * LDX + xdst[i]]) = o;
            }
        } else {
#pragma unroll
            for (int i = 0; i < UPW; ++i) *reinterpret_cast<half8v*>(&xs[8 * h * LDX + xdst[i]]) = xv[h][i];
        }
    };
    publish_x(0);
    if (M > 8) publish_x(1);

    // ---- weights -> MFMA layout, contraction ---------------------------------------------------
    const uint32_t st_w = (uint32_t)(wrow * kFlatStageRow + wchunk * 8);                  // staging write (halves)
    const uint32_t st_r = (uint32_t)(fr * kFlatStageRow + G * 8);                         // staging read
    const uint32_t xs_r = (uint32_t)((fr & (xrows - 1)) * LDX + wave * (UPW * 64) + G * 8);
    float4v acc = float4v{0.f, 0.f, 0.f, 0.f};
    auto stage = [&](int q0, int n) {
#pragma unroll
        for (int j = 0; j < n; ++j)
#pragma unroll
            for (int h = 0; h < WA; ++h)
                *reinterpret_cast<half8v*>(&wst[st_w + (j * 16 + 8 * h) * kFlatStageRow]) = wreg[q0 + j][h];
    };
    auto contract = [&](int q0, int n) {
        half8v wf[SA][2], xf[SA][2];
#pragma unroll
        for (int j = 0; j < n; ++j)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                wf[j][u] = *reinterpret_cast<const half8v*>(&wst[st_r + j * 16 * kFlatStageRow + 32 * u]);
                xf[j][u] = *reinterpret_cast<const half8v*>(&xs[xs_r + (q0 + j) * 64 + 32 * u]);
            }
#pragma unroll
        for (int j = 0; j < n; ++j)
#pragma unroll
            for (int u = 0; u < 2; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[j][u], xf[j][u], acc, 0, 0, 0);
    };
    stage(0, SA);
    __syncthreads();
    contract(0, SA);
    if (SA < UPW) {
        __builtin_amdgcn_wave_barrier();
        stage(SA, UPW - SA);
        __builtin_amdgcn_wave_barrier();
        contract(SA, UPW - SA);
    }
    __builtin_amdgcn_wave_barrier();
    // acc[r]: output column n0 + 4G + r, row fr
    *reinterpret_cast<float4v*>(&red[wave * RW + fr * 20 + 4 * G]) = acc;
    __syncthreads();
    if (writer) {
        const float* rp = &red[eml * 20 + enl];
        float4v v = *reinterpret_cast<const float4v*>(rp);
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            const float4v pw = *reinterpret_cast<const float4v*>(rp + w * RW);
            v[0] += pw[0]; v[1] += pw[1]; v[2] += pw[2]; v[3] += pw[3];
        }
        epilogue_apply<EPI>(a, eml, en, v[0], v[1], v[2], v[3], eo);
    }
}

// --------------------------------------------------------------------------------------------
// weight streaming for large layers (M <= 16 rows, tens of MB to GBs of weights per projection)
// --------------------------------------------------------------------------------------------
// Same data path as gemm_flat (whole-line loads, MFMA layout made in wave-private LDS staging
// areas, no barrier inside the K loop), but K is a loop and the activations do not fit in LDS:
//   * a workgroup of 4 waves owns 16*NF output columns; groups of UQ = 4 units (256 K values,
//     512 contiguous bytes of every weight row; 2 units with NF = 3, for the registers) are dealt
//     round-robin to the waves;
//   * a wave loads, per group, NF*UQ*2 instructions of weights and UQ*XH of activations (the
//     16 x 64 activation unit has the shape of a weight unit and takes the same road through the
//     staging areas; XH = 1 when M <= 8), for group i+1 before group i is consumed (two register
//     buffers); the scalar base pointers advance by one stride per group, so a load costs no
//     vector arithmetic at all; a group is staged two units at a time, which keeps the staging
//     space small enough for two workgroups per CU;
//   * the four partial tiles are summed through LDS once, at the end.
//
// LNS hands the statistics of the LayerNorm between two such projections from one launch to the next (GemmArgs::
// row_stats_*), so that a decode step of a large layer has no LayerNorm launch between its output projection and its first
// feed-forward projection:
//   LNS = 1 (bias + residual): the threads that write the 16 x 16*NF outputs also leave, per row, the mean and the sum of
//           squared deviations of the workgroup's columns of the rounded output;
//   LNS = 2: the workgroup first merges the producer's groups (equal sizes, so group means average; squared deviations add
//           up with the spread of the group means, taken relative to the first group's mean) into mean and 1/std per row,
//           while its first weights are in flight, and normalises every activation vector (three fused multiply-adds per
//           element) before it is staged for the matrix instructions.
// NT: the weights are loaded with the non-temporal hint (GemmArgs::read_once).  A template parameter, not a branch: the compiler
// merges the two arms of a branch whose loads differ in nothing but the hint, and drops it.
constexpr int kStreamStagedUnits = 2;
constexpr int kStreamStatsLds = 1024;                       // bytes behind the staging areas: the merged row statistics (LNS = 2)

template <int NF, int EPI, int XH, bool SL, int LNS = 0, bool NT = false>
__global__ __launch_bounds__(256) void gemm_stream(GemmArgs a) {
    static_assert(!NT || !SL, "row slices read the weights once from memory and then from the caches: plain loads");
    static_assert(LNS == 0 || !SL, "row statistics: at most 16 rows, one slice");
    static_assert(LNS != 1 || EPI == EPI_BIAS_RES, "the producer of row statistics is a bias + residual projection");
    if (SL) take_row_slice<EPI>(a);
    constexpr int UQ = NF >= 3 ? 2 : 4;                     // units per group (three or four column blocks: half as many, for the registers)
    constexpr int SU = kStreamStagedUnits;                  // units staged at a time
    constexpr int AREAS = SU * (NF + 1);                    // staging areas per wave (16 x 144 bytes each)
    extern __shared__ __attribute__((aligned(16))) unsigned char stream_smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, G = lane >> 4;
    const int wrow = lane >> 3, wchunk = lane & 7;
    const int n0 = blockIdx.x * (16 * NF);
    const int M = a.M, N = a.N, K = a.K;
    const int ngroups = K / (64 * UQ);
    half_t* wst = reinterpret_cast<half_t*>(stream_smem) + wave * (AREAS * 16 * kFlatStageRow);
    float* red = reinterpret_cast<float*>(stream_smem);

    if (a.bump_lens != nullptr && blockIdx.x == 0 && tid < a.bump_count) a.bump_lens[tid] += 1;

    // epilogue operands of the 64*NF threads that write the 16 x 16*NF outputs
    const int eml = tid / (4 * NF), enl = (tid % (4 * NF)) * 4, en = n0 + enl;
    const bool writer = tid < 64 * NF && eml < M && en < N;
    EpiOperands eo;
    if (writer) epilogue_fetch<EPI>(a, eml, en, eo);

    // per-lane byte offsets inside a group (loop invariant); the group itself moves the scalar base
    uint32_t woff[NF][2], xoff[XH];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int wr = n0 + 16 * f + 8 * h + wrow;
            wr = wr < N ? wr : N - 1;
            woff[f][h] = ((uint32_t)(wr - n0) * (uint32_t)K + wchunk * 8) * 2u;
        }
#pragma unroll
    for (int h = 0; h < XH; ++h) {
        int xr = 8 * h + wrow;
        xr = xr < M ? xr : M - 1;
        xoff[h] = ((uint32_t)xr * (uint32_t)K + wchunk * 8) * 2u;
    }
    const char* wbase = reinterpret_cast<const char*>(a.w) + (size_t)n0 * K * 2;
    const char* xbase = reinterpret_cast<const char*>(a.x);

    // Workgroups start their walk over K in eight different places (workgroups are dealt round-robin to the eight XCDs, so
    // blockIdx.x / 8 counts inside an XCD) instead of all reading the same K offset of their rows, and of the shared
    // activation rows, at the same time (rows x N x K: 16 x 36864 x 12288 166 -> 157 us, 16 x 49152 x 12288 218 -> 208,
    // 16 x 12288 x 12288 50.4 -> 47.6, 4 x 4096 x 16384 28.0 -> 21.9, 4 x 16384 x 4096 22.6 -> 21.0; K = 49152 unchanged;
    // two phases were slower than one, thirty-two slower at K = 49152).  Only the order of a column's sum depends on it.
    const int phase = (int)((((unsigned)blockIdx.x >> 3) & 7u) * (unsigned)ngroups) >> 3;
    // LNS = 2: the producer's row statistics; thread t takes row t%16 and every 16th group from t/16 on, 16 groups at a time.
    // The first 16 (all of them up to 256 groups) are requested before anything else: loads return in issue order.
    constexpr int kStatBatch = 16;
    float2v stat[LNS == 2 ? kStatBatch : 1];
    float stat0 = 0.f;                                       // the first group's mean of this thread's row
    const float2v* stat_src = reinterpret_cast<const float2v*>(a.row_stats_in) + (tid & 15);
    auto request_stats = [&](int u0) {
#pragma unroll
        for (int u = 0; u < kStatBatch; ++u) {
            const int grp = (tid >> 4) + 16 * (u0 + u);
            if (grp < a.row_stats_groups) stat[u] = stat_src[grp * 16];
        }
    };
    if constexpr (LNS == 2) {
        stat0 = stat_src[0][0];
        request_stats(0);
    }
    constexpr int GB = LNS == 2 ? UQ : 1;
    half8v wA[UQ][NF][2], xA[UQ][XH], wB[UQ][NF][2], xB[UQ][XH], gA[GB], bA[GB], gB[GB], bB[GB];
    auto request = [&](half8v (&wr)[UQ][NF][2], half8v (&xr)[UQ][XH], half8v (&gr)[GB], half8v (&br)[GB], int g) {
        g = g < ngroups ? g : ngroups - 1;                    // look-ahead past the end: a valid group, never consumed
        g += phase;                                           // this workgroup's walk starts `phase` groups into K and wraps
        g = g >= ngroups ? g - ngroups : g;
        const char* wg = wbase + (size_t)g * (UQ * 128);
        const char* xg = xbase + (size_t)g * (UQ * 128);
#pragma unroll
        for (int q = 0; q < UQ; ++q) {
            if constexpr (LNS == 2) {                         // gamma and beta of the 8 columns this lane holds of unit q
                gr[q] = *reinterpret_cast<const half8v*>(reinterpret_cast<const char*>(a.ln_gamma) + (size_t)g * (UQ * 128) + q * 128 + wchunk * 16);
                br[q] = *reinterpret_cast<const half8v*>(reinterpret_cast<const char*>(a.ln_beta) + (size_t)g * (UQ * 128) + q * 128 + wchunk * 16);
            }
#pragma unroll
            for (int h = 0; h < XH; ++h) xr[q][h] = *reinterpret_cast<const half8v*>(xg + xoff[h] + q * 128);
        }
#pragma unroll
        for (int q = 0; q < UQ; ++q)
#pragma unroll
            for (int f = 0; f < NF; ++f)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const half8v* src = reinterpret_cast<const half8v*>(wg + woff[f][h] + q * 128);
                    if constexpr (NT) wr[q][f][h] = load_once(src); else wr[q][f][h] = *src;
                }
    };
    float4v acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) acc[f] = float4v{0.f, 0.f, 0.f, 0.f};
    const uint32_t st_w = (uint32_t)(wrow * kFlatStageRow + wchunk * 8);     // staging write (halves)
    const uint32_t st_r = (uint32_t)(fr * kFlatStageRow + G * 8);            // staging read
    float ln_mu[XH], ln_rs[XH];                               // LNS = 2: mean and 1/std of this lane's activation rows
    auto consume = [&](const half8v (&wr)[UQ][NF][2], const half8v (&xr)[UQ][XH], const half8v (&gr)[GB], const half8v (&br)[GB]) {
        // area (j*(NF+1) + 0) holds the activation unit j of the round, areas +1.. its weight units
#pragma unroll
        for (int q0 = 0; q0 < UQ; q0 += SU) {
#pragma unroll
            for (int j = 0; j < SU; ++j) {
#pragma unroll
                for (int h = 0; h < XH; ++h) {
                    half8v xv = xr[q0 + j][h];
                    if constexpr (LNS == 2) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float sc = __builtin_fmaf((float)gr[q0 + j][e], ln_rs[h], 0.f);
                            const float sh = __builtin_fmaf(-ln_mu[h], sc, (float)br[q0 + j][e]);
                            xv[e] = (half_t)__builtin_fmaf((float)xv[e], sc, sh);
                        }
                    }
                    *reinterpret_cast<half8v*>(&wst[st_w + ((j * (NF + 1)) * 16 + 8 * h) * kFlatStageRow]) = xv;
                }
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        *reinterpret_cast<half8v*>(&wst[st_w + ((j * (NF + 1) + 1 + f) * 16 + 8 * h) * kFlatStageRow]) = wr[q0 + j][f][h];
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int j = 0; j < SU; ++j)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    // rows 8..15 of the activation area are stale when XH = 1: those outputs are never written
                    const half8v xf = *reinterpret_cast<const half8v*>(&wst[st_r + (j * (NF + 1)) * 16 * kFlatStageRow + 32 * u]);
#pragma unroll
                    for (int f = 0; f < NF; ++f) {
                        const half8v wf = *reinterpret_cast<const half8v*>(&wst[st_r + (j * (NF + 1) + 1 + f) * 16 * kFlatStageRow + 32 * u]);
                        acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, xf, acc[f], 0, 0, 0);
                    }
                }
            __builtin_amdgcn_wave_barrier();
        }
    };
    int g = wave;
    if (g < ngroups) request(wA, xA, gA, bA, g);
    if constexpr (LNS == 2) {
        // merge the groups: with q the first group's mean, A = sum(mean_g - q), B = sum((mean_g - q)^2), C = sum(M2_g);
        // mean = q + A/G, sum of squared deviations = C + cols * (B - A^2/G)
        float* sm = reinterpret_cast<float*>(stream_smem + 4 * AREAS * 16 * kFlatStageRow * 2);   // [4 waves][16 rows][3], then mean[16], 1/std[16]
        float A = 0.f, B = 0.f, C = 0.f;
        for (int u0 = 0; 16 * u0 < a.row_stats_groups; u0 += kStatBatch) {
            if (u0 > 0) request_stats(u0);                    // more than 256 groups: further trips, behind the first weights
#pragma unroll
            for (int u = 0; u < kStatBatch; ++u) {
                if ((tid >> 4) + 16 * (u0 + u) < a.row_stats_groups) {
                    const float dm = stat[u][0] - stat0;
                    A += dm;
                    B = __builtin_fmaf(dm, dm, B);
                    C += stat[u][1];
                }
            }
        }
        A += __shfl_xor(A, 16, kWave); B += __shfl_xor(B, 16, kWave); C += __shfl_xor(C, 16, kWave);
        A += __shfl_xor(A, 32, kWave); B += __shfl_xor(B, 32, kWave); C += __shfl_xor(C, 32, kWave);
        if (lane < 16) {
            sm[(wave * 16 + lane) * 3 + 0] = A;
            sm[(wave * 16 + lane) * 3 + 1] = B;
            sm[(wave * 16 + lane) * 3 + 2] = C;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // LDS only: the weight loads stay in flight across the barrier
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (tid < 16) {
            float At = 0.f, Bt = 0.f, Ct = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                At += sm[(w * 16 + tid) * 3 + 0];
                Bt += sm[(w * 16 + tid) * 3 + 1];
                Ct += sm[(w * 16 + tid) * 3 + 2];
            }
            const float G = (float)a.row_stats_groups, cols = (float)a.row_stats_cols;
            const float m2 = Ct + cols * fmaxf(Bt - At * At / G, 0.f);
            sm[192 + tid] = stat0 + At / G;
            sm[208 + tid] = rsqrtf(m2 / (G * cols) + a.ln_eps);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int h = 0; h < XH; ++h) {
            ln_mu[h] = sm[192 + 8 * h + wrow];
            ln_rs[h] = sm[208 + 8 * h + wrow];
        }
    }
    if (g < ngroups) {
        while (true) {
            request(wB, xB, gB, bB, g + 4);
            __builtin_amdgcn_sched_barrier(0);                // keep the look-ahead loads ahead of the arithmetic
            consume(wA, xA, gA, bA);
            g += 4;
            if (g >= ngroups) break;
            request(wA, xA, gA, bA, g + 4);
            __builtin_amdgcn_sched_barrier(0);
            consume(wB, xB, gB, bB);
            g += 4;
            if (g >= ngroups) break;
        }
    }
    // acc[f][r]: output column n0 + 16f + 4G + r, row fr.  The partial tiles go over the staging
    // space, which other waves may still be reading as theirs: barrier first.
    __syncthreads();
    constexpr int RT = 16 * (16 * NF + 4);                    // floats per wave tile: [16 rows][16*NF + 4]
#pragma unroll
    for (int f = 0; f < NF; ++f) *reinterpret_cast<float4v*>(&red[wave * RT + fr * (16 * NF + 4) + 16 * f + 4 * G]) = acc[f];
    __syncthreads();
    if (writer) {
        const float* rp = &red[eml * (16 * NF + 4) + enl];
        float4v v = *reinterpret_cast<const float4v*>(rp);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4v pw = *reinterpret_cast<const float4v*>(rp + w * RT);
            v[0] += pw[0]; v[1] += pw[1]; v[2] += pw[2]; v[3] += pw[3];
        }
        const half4v o = epilogue_apply<EPI>(a, eml, en, v[0], v[1], v[2], v[3], eo);
        if constexpr (LNS == 1) {                             // this thread's four rounded outputs: mean and squared deviations
            const float o0 = (float)o[0], o1 = (float)o[1], o2 = (float)o[2], o3 = (float)o[3];
            const float mt = 0.25f * ((o0 + o1) + (o2 + o3));
            const float d0 = o0 - mt, d1 = o1 - mt, d2 = o2 - mt, d3 = o3 - mt;
            float* sp = red + 4 * RT + tid * 2;               // behind the four waves' partial tiles
            sp[0] = mt;
            sp[1] = (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
        }
    }
    if constexpr (LNS == 1) {
        static_assert((4 * RT + 256 * 2) * 4 <= 4 * AREAS * 16 * kFlatStageRow * 2, "statistics behind the partial tiles, inside the staging space");
        __syncthreads();
        // the first of a row's 4*NF threads merges them (equal sizes: means average, squared deviations add up with the
        // spread of the means) and writes the row's pair for this workgroup
        if (writer && tid % (4 * NF) == 0) {
            const float* sp = red + 4 * RT + tid * 2;
            float ms = 0.f;
#pragma unroll
            for (int t = 0; t < 4 * NF; ++t) ms += sp[2 * t];
            const float mg = ms * (1.0f / (4 * NF));
            float m2 = 0.f;
#pragma unroll
            for (int t = 0; t < 4 * NF; ++t) {
                const float dm = sp[2 * t] - mg;
                m2 += sp[2 * t + 1] + 4.0f * dm * dm;
            }
            float* dst = a.row_stats_out + ((size_t)blockIdx.x * 16 + eml) * 2;
            dst[0] = mg;
            dst[1] = m2;
        }
    }
}

// --------------------------------------------------------------------------------------------
// dispatch
// --------------------------------------------------------------------------------------------
template <int WGM, int WGN, int BM = 256, int BN = 256, int NS = 2, int KS = 1, int SCHED = 0, bool NTS = false>
static void launch_dma64_cfg(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const int tm = (a.M + BM - 1) / BM, tn = (a.N + BN - 1) / BN;
    const dim3 grid(tm * tn), block(WGM * WGN * KS * 64);
    switch (epi) {
        case EPI_BIAS: hipLaunchKernelGGL((gemm_mfma_dma64<BM, BN, WGM, WGN, EPI_BIAS, NS, KS, SCHED, NTS>), grid, block, 0, s, a, tm, tn); break;
        case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_mfma_dma64<BM, BN, WGM, WGN, EPI_BIAS_GELU, NS, KS, SCHED, NTS>), grid, block, 0, s, a, tm, tn); break;
        case EPI_BIAS_RES: hipLaunchKernelGGL((gemm_mfma_dma64<BM, BN, WGM, WGN, EPI_BIAS_RES, NS, KS, SCHED, NTS>), grid, block, 0, s, a, tm, tn); break;
        case EPI_QKV: hipLaunchKernelGGL((gemm_mfma_dma64<BM, BN, WGM, WGN, EPI_QKV, NS, KS, SCHED, NTS>), grid, block, 0, s, a, tm, tn); break;
    }
}

template <int NF, bool LN, int NW>
static void launch_skinny_nw(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const dim3 grid((a.N + NF * 16 - 1) / (NF * 16), (a.M + 15) / 16), block(NW * 64);
    switch (epi) {
        case EPI_BIAS: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS, LN, NW>), grid, block, 0, s, a); break;
        case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS_GELU, LN, NW>), grid, block, 0, s, a); break;
        case EPI_BIAS_RES: hipLaunchKernelGGL((gemm_skinny<NF, EPI_BIAS_RES, LN, NW>), grid, block, 0, s, a); break;
        case EPI_QKV: hipLaunchKernelGGL((gemm_skinny<NF, EPI_QKV, LN, NW>), grid, block, 0, s, a); break;
    }
}
template <int NF>
static void launch_skinny_cfg(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    if (a.ln_gamma != nullptr) launch_skinny_nw<NF, true, 4>(a, epi, s);
    else launch_skinny_nw<NF, false, 4>(a, epi, s);
}
constexpr int kFlatLdsLimit = 160 * 1024;                  // LDS of one CU

static void launch_flat_kernel(void (*kernel)(GemmArgs), const GemmArgs& a, dim3 grid, dim3 block, int lds, hipStream_t s) {
    // more than 64 KB of dynamic LDS has to be allowed once per kernel and device
    if (lds > 64 * 1024) {
        static std::mutex mu;
        static std::set<std::pair<const void*, int>> allowed;
        int dev = 0;
        (void)hipGetDevice(&dev);
        std::lock_guard<std::mutex> lock(mu);
        if (allowed.insert({reinterpret_cast<const void*>(kernel), dev}).second)
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kFlatLdsLimit);
    }
    hipLaunchKernelGGL(kernel, grid, block, lds, s, a);
}

template <int NW, int UPW, int TN, bool LN, bool SL>
static void launch_flat_sl(const GemmArgs& a, Epilogue epi, int lds, hipStream_t s) {
    const dim3 grid(a.N / TN + (a.pf.blocks > 0 ? a.pf.blocks : 0), SL ? (a.M + 15) / 16 : 1), block(NW * 64);
    switch (epi) {
        case EPI_BIAS: launch_flat_kernel(gemm_flat<NW, UPW, TN, EPI_BIAS, LN, SL>, a, grid, block, lds, s); break;
        case EPI_BIAS_GELU: launch_flat_kernel(gemm_flat<NW, UPW, TN, EPI_BIAS_GELU, LN, SL>, a, grid, block, lds, s); break;
        case EPI_BIAS_RES:
            if constexpr (!LN && !SL) {
                if (a.x_splits > 1) {
                    launch_flat_kernel(gemm_flat<NW, UPW, TN, EPI_BIAS_RES, false, false, true>, a, grid, block, lds, s);
                    break;
                }
            }
            launch_flat_kernel(gemm_flat<NW, UPW, TN, EPI_BIAS_RES, LN, SL>, a, grid, block, lds, s);
            break;
        case EPI_QKV: launch_flat_kernel(gemm_flat<NW, UPW, TN, EPI_QKV, LN, SL>, a, grid, block, lds, s); break;
    }
}
template <int NW, int UPW, int TN, bool LN>
static void launch_flat_epi(const GemmArgs& a, Epilogue epi, int lds, hipStream_t s) {
    if (!LN && a.M > 16) launch_flat_sl<NW, UPW, TN, false, true>(a, epi, lds, s);     // never with the fused LayerNorm
    else launch_flat_sl<NW, UPW, TN, LN, false>(a, epi, lds, s);
}
template <int NW, int TN, bool LN>
static void launch_flat(const GemmArgs& a, int upw, Epilogue epi, int lds, hipStream_t s) {
    switch (upw) {
        case 1: launch_flat_epi<NW, 1, TN, LN>(a, epi, lds, s); break;
        case 2: launch_flat_epi<NW, 2, TN, LN>(a, epi, lds, s); break;
        case 3: launch_flat_epi<NW, 3, TN, LN>(a, epi, lds, s); break;
        default: launch_flat_epi<NW, 4, TN, LN>(a, epi, lds, s); break;
    }
}
// true when the flat kernel took the problem: a few MB of weights, K = 64 * NW * UPW with
// NW in {4, 8, 16} and UPW in 1..4, N a multiple of 16, no row maps
static bool try_flat(const GemmArgs& a, Epilogue epi, hipStream_t s, bool ask_only = false) {
    constexpr int tn8_wgs = 128;                              // fewer 16-column workgroups than this: 8-column ones
    if ((int64_t)a.N * a.K * 2 > (16 << 20) || a.N % 16 != 0 || a.K % 64 != 0) return false;
    if (a.res_row_map != nullptr || a.out_row_map != nullptr || a.tok_row_map != nullptr) return false;
    const bool ln = a.ln_gamma != nullptr;
    const int units = a.K / 64;
    auto fits = [&](int cand) { return units % cand == 0 && units / cand <= 4; };
    // fewest waves that hold K; with LN 8 waves when possible: the normalisation is vector
    // arithmetic spread over the threads
    int nw = 0;
    if (ln && fits(8)) nw = 8;
    for (int cand : {4, 8, 16})
        if (nw == 0 && fits(cand)) nw = cand;
    if (nw == 0 || (ln && nw == 16)) return false;
    const int upw = units / nw;
    const int lds = flat_lds_bytes(nw, upw, a.M <= 8 ? 8 : 16);
    if (lds > kFlatLdsLimit) return false;
    if (ask_only) return true;
    if (nw == 4) {
        // few columns: 8 per workgroup put twice the workgroups on the chip (hidden-1024 output projection: 64 -> 128
        // beside its 128 prefetch workgroups; 512 decode steps of the 24-layer stack 324.9 -> 322.6 ms, same call)
        if (ln) launch_flat<4, 16, true>(a, upw, epi, lds, s);
        else if (a.N / 16 < tn8_wgs) launch_flat<4, 8, false>(a, upw, epi, lds, s);
        else launch_flat<4, 16, false>(a, upw, epi, lds, s);
    } else if (nw == 8) {
        if (ln) launch_flat<8, 16, true>(a, upw, epi, lds, s); else launch_flat<8, 16, false>(a, upw, epi, lds, s);
    } else if (a.N / 16 < tn8_wgs) {
        launch_flat<16, 8, false>(a, upw, epi, lds, s);       // long rows, few columns: one CU cannot pull 16 rows fast enough
    } else {
        launch_flat<16, 16, false>(a, upw, epi, lds, s);
    }
    return true;
}

// LNS (see gemm_stream): 1 = leave row statistics (bias + residual), 2 = normalise the activations from them
static bool leaves_row_stats(const GemmArgs& a, Epilogue epi) { return a.row_stats_out != nullptr && epi == EPI_BIAS_RES && a.M <= 16; }
static bool takes_row_stats(const GemmArgs& a, Epilogue epi) {
    return a.row_stats_in != nullptr && a.ln_gamma != nullptr && epi == EPI_BIAS_GELU && a.M <= 16 && a.row_stats_groups >= 1 && a.row_stats_cols >= 1;
}

// at most 16 rows: one slice, with or without the non-temporal hint on the weights
template <int NF, int XH, bool NT>
static void launch_stream_rows(const GemmArgs& a, Epilogue epi, dim3 grid, dim3 block, int lds, hipStream_t s) {
    if (leaves_row_stats(a, epi)) {
        launch_flat_kernel(gemm_stream<NF, EPI_BIAS_RES, XH, false, 1, NT>, a, grid, block, lds, s);
        return;
    }
    if (takes_row_stats(a, epi)) {
        launch_flat_kernel(gemm_stream<NF, EPI_BIAS_GELU, XH, false, 2, NT>, a, grid, block, lds + kStreamStatsLds, s);
        return;
    }
    switch (epi) {
        case EPI_BIAS: launch_flat_kernel(gemm_stream<NF, EPI_BIAS, XH, false, 0, NT>, a, grid, block, lds, s); break;
        case EPI_BIAS_GELU: launch_flat_kernel(gemm_stream<NF, EPI_BIAS_GELU, XH, false, 0, NT>, a, grid, block, lds, s); break;
        case EPI_BIAS_RES: launch_flat_kernel(gemm_stream<NF, EPI_BIAS_RES, XH, false, 0, NT>, a, grid, block, lds, s); break;
        case EPI_QKV: launch_flat_kernel(gemm_stream<NF, EPI_QKV, XH, false, 0, NT>, a, grid, block, lds, s); break;
    }
}

template <int NF, int XH>
static void launch_stream(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const int lds = 4 * kStreamStagedUnits * (NF + 1) * 16 * kFlatStageRow * 2;
    const dim3 block(256);
    if (a.M > 16) {                                           // rows in slices of 16 along gridDim.y
        const dim3 grid(a.N / (16 * NF), (a.M + 15) / 16);
        switch (epi) {
            case EPI_BIAS: launch_flat_kernel(gemm_stream<NF, EPI_BIAS, XH, true>, a, grid, block, lds, s); break;
            case EPI_BIAS_GELU: launch_flat_kernel(gemm_stream<NF, EPI_BIAS_GELU, XH, true>, a, grid, block, lds, s); break;
            case EPI_BIAS_RES: launch_flat_kernel(gemm_stream<NF, EPI_BIAS_RES, XH, true>, a, grid, block, lds, s); break;
            case EPI_QKV: launch_flat_kernel(gemm_stream<NF, EPI_QKV, XH, true>, a, grid, block, lds, s); break;
        }
        return;
    }
    const dim3 grid(a.N / (16 * NF));
    if (a.read_once) launch_stream_rows<NF, XH, true>(a, epi, grid, block, lds, s);
    else launch_stream_rows<NF, XH, false>(a, epi, grid, block, lds, s);
}

// Blocks of 16 columns the streaming kernel gives a workgroup for this problem; 0: not its problem (K a multiple of 256,
// whole column tiles, and no LayerNorm unless its statistics come with the call).
static int stream_column_blocks(const GemmArgs& a, Epilogue epi) {
    if ((a.ln_gamma != nullptr && !takes_row_stats(a, epi)) || a.K % 256 != 0 || a.N % 32 != 0) return 0;
    if ((int64_t)a.M * a.K * 2 >= ((int64_t)1 << 31) || (int64_t)32 * a.K * 2 >= ((int64_t)1 << 31)) return 0;   // 32-bit lane offsets
    // With 16 rows a workgroup pulls as many activation lines out of L2 as weight lines when it owns 16
    // columns, and the stream slows down with every distinct activation line (12288 x 49152: 208 us at 1 row, 211 at
    // 8, 222 at 9, 246 at 16).  48 columns per workgroup cut that to a third: 246 -> 209 us, 12288 x 12288 60 -> 50 us,
    // 36864 x 12288 179 -> 166 us, 49152 x 12288 226 -> 219 us (16 rows each).  Taken where 48 divides N and the
    // workgroups fill the CUs evenly (N = 12288: exactly one per CU).  Sharing the activation lines between the waves of
    // a workgroup through the CU's vector cache instead (waves side by side in N, all walking the same K) changed nothing.
    const int wg48 = a.N % 48 == 0 ? a.N / 48 : 0;
    if (a.M > 4 && wg48 >= 256 && (wg48 % 256 == 0 || wg48 >= 1024)) return 3;   // (8 rows: 49152 x 12288 209 -> 205 us; 4 rows: 12288 x 4096 16.7 -> 17.8 the other way, 2 rows: no difference)
    const int wg64 = a.N % 64 == 0 ? a.N / 64 : 0;             // N without a factor of 3: 64 columns (16 rows: 16384 x 4096 25.1 -> 23.0 us,
    if (a.M > 8 && wg64 >= 256 && (wg64 % 256 == 0 || wg64 >= 1024)) return 4;   // 32768 x 8192 129 -> 114 us; nothing to gain at 4 rows)
    // Up to 8 rows otherwise 16 columns per workgroup whatever N is (32 columns, once the rule for wide outputs, lost since the
    // workgroups walk K in phases: 1 row, 36864 x 12288 168 -> 153 us, 49152 x 12288 214 -> 201, 65536 x 4096 99 -> 88;
    // 4 and 8 rows, 32768 x 8192 101 -> 93); more rows and a wide output that takes neither 48 nor 64: 32 columns.
    if (a.M <= 8) return 1;
    return a.N / 32 >= 1024 ? 2 : 1;
}

// true when the streaming kernel took the problem
static bool try_stream(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    const int nf = stream_column_blocks(a, epi);
    if (nf == 0) return false;
    const bool few = a.M <= 8;                                // at most 8 rows: one half of the activation unit
    switch (nf) {
        case 1: if (few) launch_stream<1, 1>(a, epi, s); else launch_stream<1, 2>(a, epi, s); break;
        case 2: launch_stream<2, 2>(a, epi, s); break;
        case 3: if (few) launch_stream<3, 1>(a, epi, s); else launch_stream<3, 2>(a, epi, s); break;
        default: launch_stream<4, 2>(a, epi, s); break;
    }
    return true;
}

// Row slices of the weight-streaming kernels against the tile kernels for a problem of 17 to 512 rows, from two cost
// estimates in microseconds whose constants are measured (projections of 2 to 400 MB, 17 to 1024 rows).  Slices: the
// first reads the weights at about 4 TB/s, every further one reads them again out of L2 or the memory-side cache at about
// 7.5 TB/s.  Tiles: the time does not depend on the row count while all workgroups are resident at once; it is the larger
// of the weights at about 3 TB/s and of the K loop (0.33 us per step of 64 columns, 0.23 us where two groups of waves
// share it; longer in proportion once the tiles no longer fit the chip at once).  Wide outputs with a short K go
// to the tiles from about 33 rows on, narrow outputs with a long K (the output and second feed-forward projections)
// stay with the slices for up to a few hundred rows.
static bool slices_beat_tiles(const GemmArgs& a) {
    const int slices = (a.M + 15) / 16;
    if (slices > 32) return false;
    const double w_mb = (double)a.N * a.K * 2e-6;
    const bool streams = a.K % 256 == 0 && a.N % 32 == 0;        // else the slower general kernel: 2.5 and 4.5 TB/s
    const double again = w_mb / (streams ? 7.5 : 4.5);
    const double est_slices = 2.0 + w_mb / (streams ? 4.0 : 2.5) + (slices - 1) * (again > 0.1 ? again : 0.1);
    const double wg64 = (double)((a.M + 63) / 64) * ((a.N + 63) / 64);
    const bool k_split = a.K % 128 == 0 && a.K >= 1024 && wg64 <= 256.0;     // two groups of waves share the K loop
    const double k_loop = (a.K / 64) * (k_split ? 0.23 : 0.33) * (wg64 > 768.0 ? wg64 / 768.0 : 1.0);
    const double est_tiles = 3.0 + (w_mb / 3.0 > k_loop ? w_mb / 3.0 : k_loop);
    return est_slices < est_tiles;
}

bool gemm_hands_row_stats(const GemmArgs& producer, const GemmArgs& consumer, Epilogue consumer_epi, int& groups, int& cols) {
    GemmArgs p = producer, c = consumer;
    p.row_stats_out = reinterpret_cast<float*>(16);              // any non-null value: only asked, never launched
    c.row_stats_in = reinterpret_cast<const float*>(16);
    c.row_stats_groups = c.row_stats_cols = 1;
    if (p.M < 1 || p.M > 16 || c.M != p.M || c.K != p.N || c.ln_gamma == nullptr || p.ln_gamma != nullptr || p.x_splits > 1) return false;
    if (try_flat(p, EPI_BIAS_RES, nullptr, true) || try_flat(c, consumer_epi, nullptr, true)) return false;
    const int nf = stream_column_blocks(p, EPI_BIAS_RES), nfc = takes_row_stats(c, consumer_epi) ? stream_column_blocks(c, consumer_epi) : 0;
    if (nf == 0 || p.N % (16 * nf) != 0 || nfc == 0) return false;
    // Every workgroup of the consumer merges the producer's groups before its first multiply: that pays where a workgroup
    // then streams a megabyte of weights or more and one trip brings all groups (hidden 12288 at 16 rows: 48 columns x 24 KB
    // each, 256 groups: 826 -> 818 us per step); with short-lived workgroups the launch it saves is cheaper (hidden 4096
    // at 4 rows, 16 columns x 8 KB each: 106.7 -> 108.7 us per step; hidden 12288 at 1 row, 768 groups: 638 -> 652 us).
    if ((int64_t)16 * nfc * c.K * 2 < (1 << 20) || p.N / (16 * nf) > 256) return false;
    groups = p.N / (16 * nf);
    cols = 16 * nf;
    return true;
}

bool gemm_merges_attention_ranges(const GemmArgs& a) {
    return a.M >= 1 && a.M <= 16 && a.ln_gamma == nullptr && a.d >= 8 && a.d % 8 == 0 && a.heads * a.d == a.K &&
           try_flat(a, EPI_BIAS_RES, nullptr, true);
}

// true when launch_gemm gives this problem to an MFMA tile kernel.  Only those take row strides (lda, ldy), and a
// problem that comes with strides never goes to the row slices.
static bool is_strided(const GemmArgs& a) { return (a.lda != 0 && a.lda != a.K) || (a.ldy != 0 && a.ldy != a.N); }
static bool goes_to_tile_kernel(const GemmArgs& a) {
    const bool sliced = a.M > 16 && !is_strided(a) && a.res_row_map == nullptr && a.out_row_map == nullptr && a.tok_row_map == nullptr &&
                        a.ln_gamma == nullptr && a.bump_lens == nullptr && a.pf.blocks == 0 && slices_beat_tiles(a);
    return a.M > 16 && !sliced;
}
bool gemm_takes_row_strides(const GemmArgs& a) { return a.M > 16 && a.x_splits <= 1; }

// The same problem without its first m0 rows (EPI_QKV: the prefill form, whose rows carry their sequence and position in
// tok_row_map; the decode form takes the sequence from the row number and is never cut).
static GemmArgs rows_from(const GemmArgs& a, Epilogue epi, int m0) {
    GemmArgs r = a;
    r.M = a.M - m0;
    r.x = a.x + (size_t)m0 * (a.lda ? a.lda : a.K);
    if (epi == EPI_QKV) {
        r.y = a.y + (size_t)m0 * a.hidden;
        r.tok_row_map = a.tok_row_map + m0;
        return r;
    }
    if (a.out_row_map) r.out_row_map = a.out_row_map + m0;
    else r.y = a.y + (size_t)m0 * (a.ldy ? a.ldy : a.N);
    if (a.res) {
        if (a.res_row_map) r.res_row_map = a.res_row_map + m0;
        else r.res = a.res + (size_t)m0 * a.N;
    }
    return r;
}

// One workgroup of the large-tile kernels fills a CU, so the tiles run in rounds of 256, and a launch whose last round is
// part-filled pays for more than that round: 25082 x 12288 x 49152 (18.4 rounds) 26.3 ms, 24832 rows (18.2 rounds) 26.35 ms,
// 24576 rows (18 rounds) 24.6 ms; 25082 x 36864 x 12288 (55.1 rounds) 19.1 ms, 24576 rows (54 rounds) 18.2 ms.  Where some
// number of row tiles gives whole rounds and leaves at most 16 row tiles, the launch is cut there and the rest is a launch
// of its own: small tiles below 150 large tiles' worth of rows (about 0.6 of the large tiles' rate: 506 x 12288 x 49152
// 0.85 ms), else large tiles again (506 x 36864 x 12288 0.58 ms, 506 x 49152 x 12288 0.63 ms).  Returns the rows of the
// first part, 0 for no cut.  The whole rounds are also what the tile order that lets the XCDs share operand panels
// needs (pipe::tile_of_block): 20000 x 12288 x 12288, 14.8 rounds, 4.92 ms as one launch.
static int rows_in_whole_rounds(const GemmArgs& a, Epilogue epi, int big_tiles) {
    constexpr int kCUs = 256;
    if ((epi == EPI_QKV && a.tok_row_map == nullptr) || big_tiles < 2 * kCUs || big_tiles % kCUs == 0) return 0;
    const int tm = (a.M + 255) / 256, tn = (a.N + 255) / 256;
    for (int c = tm - 1; c >= 1 && c >= tm - 16; --c) {
        if ((c * tn) % kCUs != 0) continue;
        if (a.M - c * 256 <= 16) return 0;                 // the rest would be a decode-sized problem: other kernels, no row strides
        const int rest = (tm - c) * tn;                   // large tiles' worth of rows left over
        const double rest_rounds = rest < 150 ? rest / (0.6 * kCUs) : (double)((rest + kCUs - 1) / kCUs);
        const double rounds_now = (big_tiles + kCUs - 1) / kCUs - c * tn / kCUs + 0.27;   // what the part-filled round costs on top
        return rest_rounds + 0.1 < rounds_now ? c * 256 : 0;
    }
    return 0;
}

hipError_t launch_gemm(const GemmArgs& a, Epilogue epi, hipStream_t s) {
    if (a.M <= 0) return hipSuccess;
    const bool bad_stride = (a.lda != 0 && (a.lda < a.K || a.lda % 8 != 0)) || (a.ldy != 0 && (a.ldy < a.N || a.ldy % 8 != 0));
    if (bad_stride || (is_strided(a) && (!gemm_takes_row_strides(a) || epi == EPI_QKV))) return hipErrorInvalidValue;
    if (a.x_splits > 1 && (epi != EPI_BIAS_RES || !gemm_merges_attention_ranges(a))) return hipErrorInvalidValue;
    // row statistics are between two launches of the weight-streaming kernel: asked for anywhere else, refuse
    if (a.row_stats_out != nullptr && !(leaves_row_stats(a, epi) && !try_flat(a, epi, nullptr, true) && stream_column_blocks(a, epi) != 0 &&
                                        a.N % (16 * stream_column_blocks(a, epi)) == 0)) return hipErrorInvalidValue;
    if (a.row_stats_in != nullptr && !(takes_row_stats(a, epi) && !try_flat(a, epi, nullptr, true) && stream_column_blocks(a, epi) != 0)) return hipErrorInvalidValue;
    // A few more rows than the weight-streaming kernels take at once (a decode step of more than 16 sequences, a very
    // short prompt): the same kernels with the rows cut into slices of 16 along gridDim.y, where that beats a tile kernel
    // that would run a handful of workgroups through the whole K loop (decode layer-step of the hidden-1024 layer at 32
    // sequences: 91 us with the tile kernels, 38 us so; 128 sequences: 136 -> 73 us).
    if (!goes_to_tile_kernel(a)) {
        // enough workgroups to cover the chip first, then wider slices to amortise the activations
        if (try_flat(a, epi, s)) return hipGetLastError();
        if (try_stream(a, epi, s)) return hipGetLastError();
        if (a.N >= 64 * 1024) launch_skinny_cfg<4>(a, epi, s);
        else if (a.N >= 32 * 1024) launch_skinny_cfg<2>(a, epi, s);
        else launch_skinny_cfg<1>(a, epi, s);
    } else {
        // 256x256 tiles once they cover about 60 % of the CUs, smaller tiles below that
        // (measured: 156 tiles 592 vs 514 TFLOP/s in favour of the large tiles, 112 tiles 563 vs 673 against them), and
        // never for at most 128 rows, where half of every large tile would be idle (a decode step of many sequences
        // over a very wide output, e.g. the vocabulary: 128 x 1024 x 50304 39.7 -> 30.9 us with 128x128 tiles)
        const int big_tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
        if (int m_whole = rows_in_whole_rounds(a, epi, big_tiles)) {
            // whole rounds of large tiles first, then the last few hundred rows as a problem of their own (small tiles)
            GemmArgs head = a;
            head.M = m_whole;
            hipError_t e = launch_gemm(head, epi, s);
            if (e != hipSuccess) return e;
            return launch_gemm(rows_from(a, epi, m_whole), epi, s);
        }
        if (big_tiles >= 150 && a.M > 128) {
            // Four waves with 128 x 128 each: a third less LDS read traffic per flop than eight waves of 128 x 64, and the
            // LDS of a CU -- fragment reads plus the arriving tiles -- is what the matrix pipes otherwise wait for
            // (rows x N x K, eight waves in two alternating groups -> four waves: 25082 x 49152 x 12288 1.16 -> 1.23 PFLOP/s,
            // 8192 x 16384 x 12288 1.20 -> 1.33, 2951 x 16384 x 4096 1.13 -> 1.24).  With a very long K and rows that are a
            // multiple of 32 KB apart the eight-wave kernel with the early release of the stage is ahead (25082 x 12288 x
            // 49152: 1.09 against 0.97); once the rows are 128 bytes further apart (the layer's own feed-forward buffer is
            // laid out so) both reach 1.16.
            // (that comparison was on 18.4 rounds of tiles.  On whole rounds -- which is what the cut above leaves of such a
            // launch -- the four waves are ahead at this K too: 24576 x 12288 x 49152 24.7 -> 23.7 ms, 4096 rows 3.97 -> 3.82;
            // on part-filled rounds the eight waves stay ahead: 3000 x 4096 x 32768 0.80 against 0.87 ms.)
            if (a.K >= 32768 && big_tiles % 256 != 0) launch_dma64_cfg<2, 4, 256, 256, 2, 1, 1>(a, epi, s);
            else if ((size_t)a.M * a.N * sizeof(half_t) >= kMemorySideCacheBytes) launch_dma64_cfg<2, 2, 256, 256, 2, 1, 2, true>(a, epi, s);
            else launch_dma64_cfg<2, 2, 256, 256, 2, 1, 2>(a, epi, s);
        }
        else {
            // few tiles (short prompts, narrow layers): smaller tiles put more workgroups on the chip; the K loop of
            // each is a chain of dependent steps, so what counts there is how many run side by side and how far ahead
            // the loads run: three LDS stages for the tiles that share a CU with few others
            // (rows x K x N, against two-stage register-staged tiles of the same sizes: 256 x 4096 x 4096 29.9 -> 23.8 us,
            // 2048 x 4096 x 1024 37.6 -> 28.5 us, 768 x 8192 x 2048 69.5 -> 51.9 us, 128 x 1600 x 6400 16.3 -> 11.8 us)
            const int tm = (a.M + 127) / 128;
            const int tiles128 = tm * ((a.N + 127) / 128);
            // A long K with all tiles resident at one workgroup per CU: two groups of waves per tile, each with half
            // of the K steps and LDS stages of its own, put twice the loads in flight (rows x K x N: 128 x 4096 x 4096
            // 23.8 -> 16.5 us, 96 x 16384 x 4096 101.7 -> 67.7 us, 512 x 4096 x 1024 23.3 -> 16.5 us; four groups with
            // two stages each were slower than two with three).
            const bool k_split = a.K % 128 == 0 && a.K >= 1024;
            const int wg128 = tm * ((a.N + 63) / 64), wg64 = ((a.M + 63) / 64) * ((a.N + 63) / 64);
            if (wg128 < 128) {
                if (k_split && wg64 <= 256) launch_dma64_cfg<2, 1, 64, 64, 3, 2>(a, epi, s);
                else launch_dma64_cfg<2, 1, 64, 64, 3>(a, epi, s);
            } else if (tiles128 < 256 && k_split && wg128 <= 256) launch_dma64_cfg<4, 1, 128, 64, 3, 2>(a, epi, s);
            else if (tiles128 < 256) launch_dma64_cfg<4, 1, 128, 64, 3>(a, epi, s);
            else if (tiles128 == 256) launch_dma64_cfg<2, 2, 128, 128, 3>(a, epi, s);      // one per CU
            else launch_dma64_cfg<2, 2, 128, 128>(a, epi, s);                               // two per CU
        }
    }
    return hipGetLastError();
}

}  // namespace eet
