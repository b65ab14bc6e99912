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
#include <type_traits>
#include "kernels.hpp"
#include "pipeline.hpp"

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
// CAUSAL = false is the encoder's window (Section 4, Bert layer): padding skip only, no sequence
// mask; every query tile then walks all key tiles of its sequence and only the last tile compares
// key indices (against L_b).
// The (sequence, head) pairs and their query tiles over the workgroups of a prefill launch: the tiles of a pair on one
// XCD (workgroups are dealt round-robin to the 8 XCDs; the chunk size is a multiple of 8), whose L2 then holds its K/V,
// and within a chunk of pairs the longest tiles of all its pairs first, then the next longest ... (the best balance).
// grid = (pairs, tiles) is one chunk; chunk_pairs != 0, grid = (chunks * chunk_pairs * chunk_tiles), takes the pairs
// chunk after chunk, so that the K/V of the pairs in flight stays in the memory-side cache from one tile of a pair to its
// next.  false: a pad workgroup of the last chunk.
__device__ __forceinline__ bool prefill_pair_and_tile(const AttnPrefillArgs& a, int& pair, int& tile) {
    pair = blockIdx.x;
    tile = (int)gridDim.y - 1 - (int)blockIdx.y;
    if (a.chunk_pairs != 0) {
        const int per = a.chunk_pairs * a.chunk_tiles, c = blockIdx.x / per, r = blockIdx.x - c * per;
        pair = c * a.chunk_pairs + r % a.chunk_pairs;
        tile = a.chunk_tiles - 1 - r / a.chunk_pairs;
    }
    return pair < a.batch * a.heads;
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_prefill(AttnPrefillArgs a, SeqLens lens) {
    constexpr int BQ = 128, BKV = 64;
    constexpr int LDKS = D + 8;         // K tile row stride (halfs): 16-byte reads conflict-free
    constexpr int LDVT = BKV + 4;       // V^T tile row stride: 34 dwords, so the 8-byte reads of 32 rows cover all 64 banks once
    constexpr int KVEC = BKV * D / 8 / 256;   // 16-byte vectors of K per thread per tile
    constexpr int RPT = D / 32;               // V rows per thread per tile (transposed on the way to LDS)
    constexpr int DCH = D / 8;                // 16-byte chunks per K/V row
    __shared__ __attribute__((aligned(16))) half_t Ks[BKV * LDKS];
    __shared__ __attribute__((aligned(16))) half_t Vt[D * LDVT];

    int pair, tile;
    if (!prefill_pair_and_tile(a, pair, tile)) return;
    const int b = pair / a.heads, g = pair % a.heads;
    const int L = lens.len[b];
    const int i0 = tile * BQ;
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

    const int jlast = (CAUSAL && i0 + BQ - 1 < L - 1) ? i0 + BQ - 1 : L - 1;   // last key any row of the tile sees
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
        if (CAUSAL && j0 > iw0 + 31) continue;   // whole key tile is in the future of this wave's rows

        // S^T[j][i] for 64 keys x 32 queries
        float16v st[2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[jb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk)           // the two accumulators alternate: no MFMA waits on the one before it
#pragma unroll
            for (int jb = 0; jb < 2; ++jb) {
                const half8v kf = *reinterpret_cast<const half8v*>(&Ks[(jb * 32 + li) * LDKS + kk * 16 + G * 8]);
                st[jb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[kk], st[jb], 0, 0, 0);
            }
        // st[jb][r] belongs to key j0 + jb*32 + (r/4)*8 + G*4 + r%4 and query i.
        // The attention mask is an index comparison, and only tiles that straddle the diagonal of
        // this wave's rows pay for it (wave-uniform branch).
        float tmax = -INFINITY;
        const int jmax = CAUSAL ? i : L - 1;             // last key this lane's query sees
        if (CAUSAL ? j0 + BKV - 1 > iw0 : j0 + BKV > L) {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + jb * 32 + (r >> 2) * 8 + G * 4 + (r & 3);
                    if (j > jmax) st[jb][r] = -INFINITY;
                    tmax = fmaxf(tmax, st[jb][r]);
                }
        } else {
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, st[jb][r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
        // m is the reference of the exponentials in the exp2 domain (score * c): p = 2^(s*c - m), one FMA + one
        // v_exp_f32.  It is moved (and the sum and the accumulators rescaled) only when some row's maximum has
        // grown by more than kSlack since, so p stays below 2^kSlack -- as exact in fp16 and fp32 as below 1 --
        // and the rescale is rare on any data.  m is finite from the first tile on: key 0 is visible to every row.
        constexpr float kSlack = 8.0f;
        const float tm = tmax * c;
        if (__any(tm > m + kSlack)) {
            const float m_new = fmaxf(m, tm);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            l *= alpha;
            m = m_new;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        }
        float psum = 0.f;
        half8v pf[2][2];
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[jb][r], c, -m));
                psum += p;
                pf[jb][r >> 3][r & 7] = (half_t)p;
            }
        l += psum;
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

// --------------------------------------------------------------------------------------------
// Prefill, long sequences: 256 query rows per workgroup, 8 waves of 32 rows
// --------------------------------------------------------------------------------------------
// Same arithmetic as the kernel above (S^T = K Q^T, one query per lane, O^T = V^T P^T), different
// data movement:
//  * K and V tiles go from the cache straight into LDS (global_load_lds, 16 bytes per lane, no staging
//    registers) through rings of three stages each, requested two key tiles ahead: the latency of
//    the cache is covered by two tiles of arithmetic, and there is one barrier per key tile;
//  * the tiles sit in LDS row-major, as they are in the cache: the A operand of O^T = V^T P^T is
//    fetched with the LDS transpose read (ds_read_b64_tr_b16: within 16 lanes, lane r supplies the
//    address of 4 consecutive halfs "row r"; lane l receives element l%4 of rows l/4, l/4+4, l/4+8,
//    l/4+12), so no lane transposes anything;
//  * the 16-byte chunks of a row are XOR-permuted by the row index (applied to the global address
//    of each lane when loading, to the LDS address when reading), chosen so that both the 16-byte
//    K fragment reads and the transpose reads of V touch every bank once;
//  * every LDS fragment is requested one scheduling region before the MFMA that consumes it, and
//    the scores of the next 32 keys are computed while the exponentials of the current 32 run.
// Fragment reads and their waits are inline assembly: the compiler cannot tell that an LDS read
// does not alias an in-flight global->LDS load and would drain all of them before each read.
// A wave's 32 rows start at a multiple of 32, so exactly one half tile of 32 keys -- the wave's
// last -- straddles the causal diagonal (or, without a sequence mask, the end of the sequence): it
// is the only one that compares indices.  Waves whose rows end before the workgroup's last key
// tile keep loading and synchronising but skip the arithmetic; the row blocks are dealt to the
// waves so that the two waves of a SIMD (w and w+4) always sum to the same amount of work.
// LDS transpose read (gfx950): within 16 lanes, lane r supplies the address of 4 consecutive halfs "row r"; lane l
// receives element l%4 of rows l/4, l/4+4, l/4+8, l/4+12.
__device__ __forceinline__ half4v lds_read_tr16(const char* p) {
    typedef short short4v __attribute__((ext_vector_type(4)));
    const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(half4v, v);
}

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds + 16*l (the LDS base
// must be wave-uniform).  Kept out of the templates: the builtin only exists for the device.
__device__ __forceinline__ void load_lds_16B(const char* gptr, char* lds) {
    __builtin_amdgcn_global_load_lds(gptr, lds, 16, 0, 0);
}
template <int N>
__device__ __forceinline__ void wait_lds() {
    static_assert(N == 0 || N == 4 || N == 8 || N == 16, "add the count");
    if (N == 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (N == 4) asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory");
    if (N == 8) asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
    if (N == 16) asm volatile("s_waitcnt lgkmcnt(15)" ::: "memory");   // the counter saturates at 15: one read more than needed is waited for
}
template <int N>
__device__ __forceinline__ void wait_vmem() {
    static_assert(N == 2 || N == 4, "add the count");
    if (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    if (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
}
// lane ^ 32 maximum without the LDS: v_permlane32_swap exchanges the upper half of its first operand
// with the lower half of its second, so the two results hold, for every lane, its own value and its partner's.
// The two elements are copied into scalars before the bit casts: __builtin_bit_cast applied to the vector element
// r[1] directly reads element 0 with this compiler, which silently turned the maximum into "the value of the lower
// lane" (a reference of the exponentials that ignored half of each row's keys: exact results until a row's scores
// span more than the 16 bits of headroom fp16 has above one, then infinities).
__device__ __forceinline__ float max_xor32(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}

// Executor of pipe::attn_kv_loop for the kernel below: the tile loads and the arithmetic of a step are the kernel's
// own lambdas, the waits and the barrier are the instructions themselves.  PAIR = load instructions of one
// load_k + load_v pair of a wave.
template <int PAIR, class LoadK, class LoadV, class First, class Step>
struct AttnRingExec {
    LoadK& load_k_;
    LoadV& load_v_;
    First& first_;
    Step& step_;
    __device__ __forceinline__ void load_k(int tile, int stage) { load_k_(tile, stage); }
    __device__ __forceinline__ void load_v(int tile, int stage) { load_v_(tile, stage); }
    __device__ __forceinline__ void wait_loads_but_newest_pair() { wait_vmem<PAIR>(); }
    __device__ __forceinline__ void wait_loads_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
    __device__ __forceinline__ void barrier() { __builtin_amdgcn_s_barrier(); }
    __device__ __forceinline__ void first_scores() { first_(); }
    __device__ __forceinline__ void step(int jt, int v_stage, int k_stage) { step_(jt, v_stage, k_stage); }
    __device__ __forceinline__ void wait_reads() { wait_lds<0>(); }
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(512) void attn_prefill_wide(AttnPrefillArgs a, SeqLens lens) {
    constexpr int BQ = 256, WQ = 32, BKV = 64, NWAVE = 8;
    constexpr int ROWB = D * 2;                  // bytes of a K / V row
    constexpr int TILEB = BKV * ROWB;            // bytes of a key tile
    constexpr int CPR = ROWB / 16;               // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;                // rows one wave-level load instruction covers (1 KB of LDS)
    constexpr int NV = TILEB / 1024 / NWAVE;     // load instructions per wave per tile
    constexpr int KK = D / 16, DB = D / 32;
    __shared__ __attribute__((aligned(1024))) char Ks[3][TILEB];
    __shared__ __attribute__((aligned(1024))) char Vs[3][TILEB];

    int pair, tile;
    if (!prefill_pair_and_tile(a, pair, tile)) return;
    const int b = pair / a.heads, g = pair % a.heads;
    const int L = lens.len[b];
    const int i0 = tile * BQ;
    if (i0 >= L) return;                                          // pad queries are never visited
    int row0 = b * a.S;
    if (a.packed) {
        row0 = 0;
        for (int k = 0; k < b; ++k) row0 += lens.len[k];
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, G = lane >> 5;
    const int iw0 = i0 + (wave < 4 ? wave : 11 - wave) * WQ;      // SIMD s hosts row blocks s and 7-s
    const int i = iw0 + li;                                       // this lane's query

    const int last_key = (CAUSAL && i0 + BQ - 1 < L - 1) ? i0 + BQ - 1 : L - 1;
    const int nt_wg = last_key / BKV + 1;                         // key tiles the workgroup stages
    // halves (32 keys) this wave uses; the last one is the only one with hidden keys
    const int nh_w = iw0 >= L ? 0 : (CAUSAL ? iw0 / 32 + 1 : (L + 31) / 32);

    // Q^T fragments (B operand): query i, depth kk*16 + G*8 .. +8
    half8v qf[KK];
    {
        const half_t* qp = a.q + (int64_t)(row0 + (i < L ? i : L - 1)) * a.hidden + g * D + G * 8;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) qf[kk] = *reinterpret_cast<const half8v*>(qp + kk * 16);
    }
    const int64_t head_off = ((int64_t)b * a.heads + g) * a.capacity * D;
    const char* kbase = reinterpret_cast<const char*>(a.k_cache + head_off);
    const char* vbase = reinterpret_cast<const char*>(a.v_cache + head_off);

    // Tile loads.  Load instruction v of this wave fills LDS bytes [(wave*NV + v)*1024, +1024) of a stage:
    // lane -> row (wave*NV + v)*RPI + lane/CPR, position lane%CPR, which receives the source chunk
    // position ^ swizzle(row).  Rows past the sequence are clamped: slots >= L of the cache are never read.
    int ld_row[NV];
    uint32_t ld_k[NV], ld_v[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int row = (wave * NV + v) * RPI + lane / CPR, pos = lane % CPR;
        const int swk = D == 128 ? (row & 15) : ((row >> 1) & 7);
        const int swv = D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
        ld_row[v] = row;
        ld_k[v] = (uint32_t)((pos ^ swk) * 16);
        ld_v[v] = (uint32_t)((pos ^ swv) * 16);
    }
    auto load_k = [&](int jt, int st) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int key = jt * BKV + ld_row[v];
            key = key < L ? key : L - 1;
            load_lds_16B(kbase + ((uint32_t)key * ROWB + ld_k[v]), &Ks[st][(wave * NV + v) * 1024]);
        }
    };
    auto load_v = [&](int jt, int st) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int key = jt * BKV + ld_row[v];
            key = key < L ? key : L - 1;
            load_lds_16B(vbase + ((uint32_t)key * ROWB + ld_v[v]), &Vs[st][(wave * NV + v) * 1024]);
        }
    };

    // fragment addresses (LDS byte addresses relative to stage 0 of the ring)
    unsigned kaddr[KK];     // K row li (+ jb*32 rows), chunk kk*2 + G
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int sw = D == 128 ? (li & 15) : ((li >> 1) & 7);
        kaddr[kk] = (unsigned)(uintptr_t)&Ks[0][0] + li * ROWB + (((kk * 2 + G) ^ sw) * 16);
    }
    unsigned vaddr[DB];     // transpose read: this lane supplies key G*4 + (li%16)/4 (+ offset), 4 halfs at dv db*32 + (li/16)*16 + (li%4)*4
    {
        const int lb = li & 15, blk = li >> 4;
        const int sw = D == 128 ? (((lb >> 2) & 3) << 2) : (((lb >> 3) & 1) << 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int cc = db * 4 + blk * 2 + ((lb & 3) >> 1);
            vaddr[db] = (unsigned)(uintptr_t)&Vs[0][0] + (G * 4 + (lb >> 2)) * ROWB + ((cc ^ sw) * 16) + (lb & 1) * 8;
        }
    }

    float16v o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m = -INFINITY, l = 0.f, alpha = 1.f;
    bool rescale = false;
    constexpr float kSlack = 8.0f;
    const float c = rsqrtf((float)D) * kLog2e;

    // Pipeline over halves of 32 keys, h = 2*tile + jb.  Scores of half h: st[r] belongs to key
    // jb*32 + (r/4)*8 + G*4 + r%4 of the tile and query i.  One step handles half h in two
    // scheduling regions (fenced, so that the fragment reads issued in a region stay there: an LDS
    // read takes longer than the MFMA it feeds):
    //   region 1: LDS: V^T fragments of half h requested (transpose reads)
    //             matrix cores: scores of half h+1 (K fragments requested one region earlier)
    //             vector units: p = 2^(s*c - m) of half h, row sum, conversion to P^T (B-operand layout)
    //   region 2: LDS: K fragments of half h+2 requested
    //             matrix cores: O^T += V^T P^T of half h
    //             vector units: window test (last half only) and running maximum of half h+1
    // followed by the rescale of the accumulators in the rare case that some row's maximum moved.
    half8v kf[KK];                // K fragments (A operand): key row jb*32 + li, depth kk*16 + G*8 .. +8
    auto read_k = [](half8v (&dst)[KK], const unsigned (&ka)[KK], auto jb) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[kk]) : "v"(ka[kk]), "n"(decltype(jb)::value * 32 * ROWB) : "memory");
    };
    auto landed_k = [&]() __attribute__((always_inline)) {     // after a wait: the fragments are now defined
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) asm volatile("" : "+v"(kf[kk]));
    };
    auto scores = [&](float16v& st) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) st = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], qf[kk], st, 0, 0, 0);
    };
    // Window test + running maximum of one half.  The mask is an index comparison on the lane's own
    // indices (Algorithm 1); nothing is read for it.  The maximum lives in the exp2 domain (score * c)
    // and is finite from the first half on: key 0 is visible to every row.
    auto row_max = [&](float16v& st, int j0, auto masked) __attribute__((always_inline)) {
        if constexpr (decltype(masked)::value) {
            const int jmax = CAUSAL ? i : L - 1;                  // last key this lane's query sees
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + (r >> 2) * 8 + G * 4 + (r & 3);
                if (j > jmax) st[r] = -INFINITY;
            }
        }
        float tmax = st[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, st[r]);
        tmax = max_xor32(tmax) * c;
        // m is the reference of the exponentials, not necessarily the maximum: it is moved (and the sum and the
        // accumulators rescaled) only when some row's maximum has grown by more than kSlack since, so p stays
        // below 2^kSlack -- exact in fp16 and fp32 all the same -- and the rescale is rare on any data.
        rescale = __any(tmax > m + kSlack);
        if (rescale) {
            const float m_new = fmaxf(m, tmax);
            alpha = __builtin_amdgcn_exp2f(m - m_new);
            l *= alpha;
            m = m_new;
        }
    };
    auto half_step = [&](float16v& cur, float16v& nxt, const unsigned (&va)[DB], auto jb, const unsigned (&ka2)[KK], int j0_next,
                         auto has_next, auto mask_next, auto prefetch) __attribute__((always_inline)) {
        // ---- region 1
        half4v vlo[2][DB], vhi[2][DB];
        constexpr int JB = decltype(jb)::value;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vlo[hf][db]) : "v"(va[db]), "n"((JB * 32 + hf * 16) * ROWB) : "memory");
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vhi[hf][db]) : "v"(va[db]), "n"((JB * 32 + hf * 16 + 8) * ROWB) : "memory");
            }
        if constexpr (decltype(has_next)::value) {
            wait_lds<4 * DB>();                                   // the K fragments requested one region ago
            landed_k();
            scores(nxt);
        }
        half8v pf[2];             // slot s of pf[hf] <-> key jb*32 + hf*16 + (s/4)*8 + G*4 + s%4
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[r], c, -m));
            psum += p;
            pf[r >> 3][r & 7] = (half_t)p;
        }
        l += psum;
        __builtin_amdgcn_sched_barrier(0);
        // ---- region 2
        if constexpr (decltype(prefetch)::value) {
            read_k(kf, ka2, jb);
            wait_lds<KK>();                                       // the V fragments; the K reads stay in flight
        } else {
            wait_lds<0>();
        }
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                asm volatile("" : "+v"(vlo[hf][db]), "+v"(vhi[hf][db]));
                const half8v vf = __builtin_shufflevector(vlo[hf][db], vhi[hf][db], 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[hf], o[db], 0, 0, 0);
            }
        if constexpr (decltype(has_next)::value) row_max(nxt, j0_next, mask_next);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(has_next)::value) {
            if (rescale) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            }
        }
    };
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    // half h of the wave: cur holds its scores; the K fragments of half h+1 have been requested
    auto wave_half = [&](int h, auto jb, float16v& cur, float16v& nxt, const unsigned (&va)[DB], const unsigned (&ka2)[KK]) __attribute__((always_inline)) {
        const int j0_next = (h + 1) * 32;
        if (h + 2 < nh_w) half_step(cur, nxt, va, jb, ka2, j0_next, yes, no, yes);
        else if (h + 2 == nh_w) half_step(cur, nxt, va, jb, ka2, j0_next, yes, yes, no);   // the next half is the last: its keys are tested
        else if (h + 1 == nh_w) half_step(cur, nxt, va, jb, ka2, j0_next, no, no, no);
    };
    constexpr std::integral_constant<int, 0> jb0{};
    constexpr std::integral_constant<int, 1> jb1{};

    // Rings: tile t lives in stage t%3.  Which stage is loaded, read, waited for and released when is
    // pipe::attn_kv_loop (pipeline.hpp), shared with the host-side audit of the hand-over; the lambdas below are
    // the instructions of its steps.
    float16v sa, sb;
    auto first_scores = [&]() __attribute__((always_inline)) {
        if (nh_w > 0) {
            read_k(kf, kaddr, jb0);
            wait_lds<0>();
            landed_k();
            scores(sa);
            if (nh_w == 1) row_max(sa, 0, yes);
            else row_max(sa, 0, no);                      // alpha = 0 and the accumulators are zero: nothing to rescale
            if (nh_w > 1) read_k(kf, kaddr, jb1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto step = [&](int jt, int v_stage, int k_stage) __attribute__((always_inline)) {
        unsigned ka2[KK], va[DB];                         // fragment addresses in the stages of K(jt+1) and V(jt)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) ka2[kk] = kaddr[kk] + k_stage * TILEB;
#pragma unroll
        for (int db = 0; db < DB; ++db) va[db] = vaddr[db] + v_stage * TILEB;
        wave_half(2 * jt, jb0, sa, sb, va, ka2);          // requests the K fragments of half 2*jt+2: tile jt+1, jb 0
        wave_half(2 * jt + 1, jb1, sb, sa, va, ka2);      // ... of half 2*jt+3: tile jt+1, jb 1
    };
    AttnRingExec<2 * NV, decltype(load_k), decltype(load_v), decltype(first_scores), decltype(step)> ring{load_k, load_v, first_scores, step};
    pipe::attn_kv_loop(ring, nt_wg);

    l += __shfl_xor(l, 32, kWave);
    if (i >= L) return;
    const float inv = 1.0f / l;
    half_t* op = a.ctx + (int64_t)(row0 + i) * a.hidden + g * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            half4v t;
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = (half_t)(o[db][rg * 4 + e] * inv);
            *reinterpret_cast<half4v*>(op + db * 32 + rg * 8 + G * 4) = t;
        }
}

// K/V of the pairs of one chunk of a prefill launch (16 to 48 pairs: two to six per XCD)
constexpr size_t kChunkKvBytes = (size_t)64 << 20;
hipError_t launch_attention_prefill(const AttnPrefillArgs& a, const SeqLens& lens, hipStream_t s) {
    // 256-row kernel for heads of 128 and prompts beyond 512 tokens (measured, one call: equal to the 128-row kernel
    // from 512 to 1024 tokens, 15-20 % ahead from 2048 on, 6-15 % behind up to 512, where twice as many workgroups
    // matter more than the deeper pipeline); heads of 64 have half the matrix work per score, and the 128-row kernel
    // (softmax over 64 keys at a time) is the faster one there.
    const bool wide = a.d == 128 && a.max_len > 512;
    const int bq = wide ? 256 : 128;
    const dim3 grid(a.heads * a.batch, (a.max_len + bq - 1) / bq), block(wide ? 512 : 256);
    // In chunks of pairs once the K/V of the launch is more than the memory-side cache holds: with the tiles of all
    // pairs in turn, a pair's K/V then comes from HBM again for every one of its tiles (16 prompts of 1024-2048
    // tokens, 96 heads: 6.3 GB fetched for 1.2 GB of K/V and 0.6 GB of Q).  TFLOP/s by pairs per chunk, one call
    // (none / 8 / 16 / 32 / 48 / 96 / 192): those prompts 577-604 / 622 / 680 / 703 / 689 / 677 / 669; 16 prompts of
    // 2048-4096 tokens, 32 heads 711-734 / 811 / 824 / 848 / 831 / 820 / 806; 16 of 512-1024 tokens, 96 heads 414-448
    // / 378 / 470 / 504 / 498 / 508 / 494; 4 prompts of 8192-16384 tokens, 32 heads (none / 8 / 16 / 32 / 64) 922 / 1011 /
    // 1013 / 997 / 950; the 128-row kernel (none / 8 / 16 / 32 / 48 / 96): 128 prompts of 256-512 tokens, 32 heads of 64
    // 222-260 / 262 / 296 / 306 / 307 / 308, 16 of 1024-2048 tokens, 64 heads of 64 492-538 / 576 / 594 / 601 / 593 / 580;
    // below the cache's size chunks gain nothing (4 prompts of 1024-2048 tokens, 96 heads, 303 MB:
    // 601-645 / 590 / 651 / 672 / 684 / 685 / 663; 167 MB: 640-705 / 556 / 639 / 696 / 691 / 692 / 712).
    AttnPrefillArgs w = a;
    size_t kv_bytes = 0;
    for (int b = 0; b < a.batch; ++b) kv_bytes += (size_t)lens.len[b] * a.heads * a.d * 2 * sizeof(half_t);
    const int pairs = (int)grid.x;
    int chunk = 0;
    if (kv_bytes > kMemorySideCacheBytes) {
        chunk = (int)(kChunkKvBytes / (kv_bytes / pairs)) / 8 * 8;
        chunk = chunk < 16 ? 16 : chunk > 48 ? 48 : chunk;
    }
    w.chunk_pairs = chunk >= pairs ? 0 : chunk;
    w.chunk_tiles = (int)grid.y;
    const dim3 wgrid = w.chunk_pairs ? dim3((pairs + chunk - 1) / chunk * chunk * grid.y) : grid;
    if (wide) {
        if (a.causal) hipLaunchKernelGGL((attn_prefill_wide<128, true>), wgrid, block, 0, s, w, lens);
        else hipLaunchKernelGGL((attn_prefill_wide<128, false>), wgrid, block, 0, s, w, lens);
    } else if (a.causal) {
        if (a.d == 128) hipLaunchKernelGGL((attn_prefill<128, true>), wgrid, block, 0, s, w, lens);
        else hipLaunchKernelGGL((attn_prefill<64, true>), wgrid, block, 0, s, w, lens);
    } else {
        if (a.d == 128) hipLaunchKernelGGL((attn_prefill<128, false>), wgrid, block, 0, s, w, lens);
        else hipLaunchKernelGGL((attn_prefill<64, false>), wgrid, block, 0, s, w, lens);
    }
    return hipGetLastError();
}

// ============================================================================================
// Unfused, paper-form attention: scores = Q K^T, Algorithm 1 as a kernel of its own (rowops), O = P V
// ============================================================================================
// The form Section 2.1 describes: the scores of a prompt are materialised as [batch, heads, S, S], the
// mask-free softmax runs in place on them, and a second contraction applies them to V.  Padding is skipped in
// all three steps: tiles of pad queries, of keys past the sequence and of keys in the future of every query of
// the tile are neither computed nor read; inside the tiles that are, the softmax kernel decides entry by entry.
//
// Scores: one 128 x 128 tile per workgroup, 2 x 2 waves of 64 x 64.  The contraction depth is the head size, so
// every operand element is used by one wave exactly once: fragments come straight from global memory in MFMA
// layout.  Computed transposed (keys as the A operand) so that a lane ends up with 4 consecutive keys of one query.
template <int D>
__global__ __launch_bounds__(256) void attn_scores(AttnPrefillArgs a, SeqLens lens, half_t* scores) {
    constexpr int KK = D / 16;
    const int b = blockIdx.x / a.heads, g = blockIdx.x % a.heads;
    const int L = lens.len[b];
    const int i0 = blockIdx.y * 128, j0 = blockIdx.z * 128;
    if (i0 >= L || j0 >= L || j0 > i0 + 127) return;          // pad queries, pad keys, keys no query of the tile sees
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, G = lane >> 5;
    const int iw = i0 + (wave >> 1) * 64, jw = j0 + (wave & 1) * 64;
    const half_t* kbase = a.k_cache + ((int64_t)b * a.heads + g) * a.capacity * D;
    const half_t* qbase = a.q + (int64_t)b * a.S * a.hidden + g * D;

    half8v kf[2][KK], qf[2][KK];
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        int j = jw + f * 32 + li, i = iw + f * 32 + li;
        j = j < L ? j : L - 1;                                  // slots >= L of the cache and pad rows of q are never read
        i = i < L ? i : L - 1;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            kf[f][kk] = *reinterpret_cast<const half8v*>(kbase + (int64_t)j * D + kk * 16 + G * 8);
            qf[f][kk] = *reinterpret_cast<const half8v*>(qbase + (int64_t)i * a.hidden + kk * 16 + G * 8);
        }
    }
    half_t* out = scores + ((int64_t)b * a.heads + g) * a.S * a.S;
#pragma unroll
    for (int fi = 0; fi < 2; ++fi) {
        const int i = iw + fi * 32 + li;
#pragma unroll
        for (int fj = 0; fj < 2; ++fj) {
            float16v acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[fj][kk], qf[fi][kk], acc, 0, 0, 0);
            if (i >= L) continue;
            // acc[r]: key jw + fj*32 + (r/4)*8 + G*4 + r%4, query i.  Entries past the row's window hold raw scores;
            // Algorithm 1 overwrites them.
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int j = jw + fj * 32 + rg * 8 + G * 4;
                if (j >= a.S) continue;                          // S is a multiple of 8: a group of 4 is inside or outside
                half4v t;
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = (half_t)acc[rg * 4 + e];
                *reinterpret_cast<half4v*>(out + (int64_t)i * a.S + j) = t;
            }
        }
    }
}

// O = P V from materialised probabilities.  Workgroup = 4 waves = 128 query rows, wave w rows 32w..32w+31; key tiles
// of 64: V row-major in LDS (chunks XOR-permuted by the row, transpose reads give the A operand of O^T = V^T P^T), P^T
// fragments straight from the probability rows (a lane owns one query and reads 8 consecutive keys).  Keys past
// the diagonal tile are not visited; inside it the probabilities of hidden keys are the zeros Algorithm 1 wrote.
template <int D>
__global__ __launch_bounds__(256) void attn_apply(AttnPrefillArgs a, SeqLens lens, const half_t* probs) {
    constexpr int BQ = 128, BKV = 64, ROWB = D * 2, CPR = ROWB / 16, DB = D / 32;
    constexpr int NV = BKV * CPR / 256;                         // 16-byte chunks each thread stages per tile
    __shared__ __attribute__((aligned(1024))) char Vs[BKV * ROWB];
    const int b = blockIdx.x / a.heads, g = blockIdx.x % a.heads;
    const int L = lens.len[b];
    const int i0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * BQ; // longest query tiles first
    if (i0 >= L) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, G = lane >> 5;
    const int iw0 = i0 + wave * 32, i = iw0 + li;
    const char* vbase = reinterpret_cast<const char*>(a.v_cache + ((int64_t)b * a.heads + g) * a.capacity * D);
    const half_t* prow = probs + (((int64_t)b * a.heads + g) * a.S + (i < L ? i : L - 1)) * a.S;

    const int s_row = tid / CPR, s_pos = tid % CPR;
    const int swv = D == 128 ? ((s_row & 3) << 2) : (((s_row >> 1) & 1) << 2);
    const uint32_t v_src = (uint32_t)((s_pos ^ swv) * 16);
    unsigned vaddr[DB];     // transpose read: this lane supplies key G*8 + (li%16)/4 (+ offset), 4 halfs at dv db*32 + (li/16)*16 + (li%4)*4
    {
        const int lb = li & 15, blk = li >> 4;
        const int sw = D == 128 ? (((lb >> 2) & 3) << 2) : (((lb >> 3) & 1) << 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int cc = db * 4 + blk * 2 + ((lb & 3) >> 1);
            vaddr[db] = (G * 8 + (lb >> 2)) * ROWB + ((cc ^ sw) * 16) + (lb & 1) * 8;
        }
    }
    float16v o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;

    const int last_key = i0 + BQ - 1 < L - 1 ? i0 + BQ - 1 : L - 1;
    const int ntiles = last_key / BKV + 1;
    for (int jt = 0; jt < ntiles; ++jt) {
        const int j0 = jt * BKV;
        half8v rv[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            int key = j0 + v * (256 / CPR) + s_row;
            key = key < L ? key : L - 1;                        // probabilities of keys >= L are zero; their values must be finite
            rv[v] = *reinterpret_cast<const half8v*>(vbase + ((uint32_t)key * ROWB + v_src));
        }
        __syncthreads();                                        // everyone is done reading the previous tile
#pragma unroll
        for (int v = 0; v < NV; ++v) *reinterpret_cast<half8v*>(&Vs[(v * 256 + tid) * 16]) = rv[v];
        __syncthreads();
        if (j0 > iw0 + 31 || iw0 >= L) continue;                // whole key tile is in the future of this wave's rows
#pragma unroll
        for (int kk = 0; kk < BKV / 16; ++kk) {
            // keys j0 + kk*16 + G*8 .. +8 of this lane's query (row stride S is a multiple of 8: 16-byte aligned)
            const half8v pf = j0 + kk * 16 + G * 8 < a.S ? *reinterpret_cast<const half8v*>(prow + j0 + kk * 16 + G * 8)
                                                         : half8v{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const char* vp = Vs + vaddr[db] + kk * 16 * ROWB;
                const half4v lo = lds_read_tr16(vp);
                const half4v hi = lds_read_tr16(vp + 4 * ROWB);
                const half8v vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, o[db], 0, 0, 0);
            }
        }
    }
    if (i >= L) return;
    half_t* op = a.ctx + ((int64_t)b * a.S + i) * a.hidden + g * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            half4v t;
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = (half_t)o[db][rg * 4 + e];
            *reinterpret_cast<half4v*>(op + db * 32 + rg * 8 + G * 4) = t;
        }
}

hipError_t launch_attention_scores(const AttnPrefillArgs& a, const SeqLens& lens, half_t* scores, hipStream_t s) {
    const int tiles = (a.max_len + 127) / 128;
    const dim3 grid(a.heads * a.batch, tiles, tiles), block(256);
    if (a.d == 128) hipLaunchKernelGGL(attn_scores<128>, grid, block, 0, s, a, lens, scores);
    else hipLaunchKernelGGL(attn_scores<64>, grid, block, 0, s, a, lens, scores);
    return hipGetLastError();
}

hipError_t launch_attention_apply(const AttnPrefillArgs& a, const SeqLens& lens, const half_t* probs, hipStream_t s) {
    const dim3 grid(a.heads * a.batch, (a.max_len + 127) / 128), block(256);
    if (a.d == 128) hipLaunchKernelGGL(attn_apply<128>, grid, block, 0, s, a, lens, probs);
    else hipLaunchKernelGGL(attn_apply<64>, grid, block, 0, s, a, lens, probs);
    return hipGetLastError();
}

// ============================================================================================
// Decode: one query per (sequence, head), K and V streamed once from HBM
// ============================================================================================
// grid = (splits, heads, batch); a workgroup of NW waves owns one contiguous range of keys and
// walks it in blocks of BK keys dealt round-robin to the waves, so the waves stream one
// region together.  The work per (sequence, head) is small and has no reuse: what sets the speed
// is memory-level parallelism and the number of instructions a wave issues, not arithmetic, so
// there is no MFMA here.  A key row (d halves) is spread over d/8 adjacent lanes, 16 bytes each:
// every load instruction reads 1 KB of contiguous cache (whole 128-byte lines), K and V rows are
// addressed by the same 32-bit offset, and the loads of block i+1 are issued before block i is
// consumed.  q.k is four 2-way dot instructions per lane plus a lane-exchange reduction inside
// the row's lanes; every lane then owns the softmax weight of its key and multiplies it into its
// own 8 values of that key's V row.  Each group of d/8 lanes keeps its own running (max, sum,
// values) over the keys it has seen (rescaled once per block); groups, then waves, are merged at
// the end.  The padding offset is the loop bound: slots >= n_b are never used (the tail of the
// last block re-reads the last valid row with weight zero).
//
// With more than one range per (sequence, head) each workgroup writes a partial (max, sum,
// values) and attn_decode_combine merges them.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// NT: K and V rows are loaded with the non-temporal hint (AttnDecodeArgs::read_once); a template parameter because the
// compiler merges the arms of a branch whose loads differ in nothing but the hint, and drops it.
template <int D, int NW, bool NT>
__global__ __launch_bounds__(NW * 64) void attn_decode(AttnDecodeArgs a) {
    constexpr int LPK = D / 8;           // lanes per key row (8 or 16)
    constexpr int KPI = 64 / LPK;        // key rows per load instruction (8 or 4)
    constexpr int U = 8;                 // load instructions (of K, and of V) per block
    constexpr int BK = U * KPI;          // keys per block (64 or 32)
    constexpr float kEmpty = -1e30f;     // running maximum before any key: finite, so exp2(m - m) is 1, not NaN
    __shared__ float sm_m[NW], sm_l[NW];
    __shared__ float sm_acc[NW][D];

    const int sp = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kslot = lane / LPK, chunk = lane % LPK;
    int n = a.lens[b] + a.len_bias;                      // visible keys
    n = n < 0 ? 0 : (n > a.capacity ? a.capacity : n);   // whatever the device-side length says, never outside the pair's slots
    const int splits = a.splits;
    int per = (n + splits - 1) / splits;
    per = (per + 15) & ~15;
    const int c0 = sp * per;
    const int c1 = (c0 + per < n) ? c0 + per : n;        // may be <= c0: empty range of a short sequence
    const int64_t bh = (int64_t)b * a.heads + g;
    // uniform bases + one 32-bit per-lane byte offset shared by the K and the V load of a row
    const char* kbase = reinterpret_cast<const char*>(a.k_cache + bh * a.capacity * D);
    const char* vbase = reinterpret_cast<const char*>(a.v_cache + bh * a.capacity * D);
    const uint32_t lane_off = (uint32_t)chunk * 16u;

    const half8v qv = *reinterpret_cast<const half8v*>(a.q + bh * D + chunk * 8);
    half2v q2[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) q2[e] = half2v{qv[2 * e], qv[2 * e + 1]};

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    float m = kEmpty, l = 0.f;
    const float c = rsqrtf((float)D) * kLog2e;

    auto request = [&](half8v (&kf)[U], half8v (&vf)[U], int j0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int row = j0 + u * KPI + kslot;
            row = row < c1 ? row : c1 - 1;                // weight zero in consume()
            const uint32_t off = (uint32_t)row * (uint32_t)(D * 2) + lane_off;
            if constexpr (NT) {
                kf[u] = load_once(reinterpret_cast<const half8v*>(kbase + off));
                vf[u] = load_once(reinterpret_cast<const half8v*>(vbase + off));
            } else {
                kf[u] = *reinterpret_cast<const half8v*>(kbase + off);
                vf[u] = *reinterpret_cast<const half8v*>(vbase + off);
            }
        }
    };
    auto consume = [&](const half8v (&kf)[U], const half8v (&vf)[U], int j0) {
        float sc[U], mx = kEmpty;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) d = __builtin_amdgcn_fdot2(half2v{kf[u][2 * e], kf[u][2 * e + 1]}, q2[e], d, false);
            d += dpp_f<0xb1>(d);                          // lane ^ 1
            d += dpp_f<0x4e>(d);                          // lane ^ 2
            d += dpp_f<0x141>(d);                         // the other quad of 8
            if (LPK == 16) d += dpp_f<0x140>(d);          // the other half of 16
            sc[u] = (j0 + u * KPI + kslot < c1) ? d * c : -INFINITY;
            mx = fmaxf(mx, sc[u]);
        }
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = __builtin_amdgcn_exp2f(sc[u] - m_new);
            l += p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(p, (float)vf[u][e], acc[e]);
        }
        m = m_new;
    };
    // blocks wave, wave + 4, ... of the range; two register buffers, loop unrolled by two
    half8v kA[U], vA[U], kB[U], vB[U];
    int j0 = c0 + wave * BK;
    if (j0 < c1) {
        request(kA, vA, j0);
        while (true) {
            request(kB, vB, j0 + NW * BK);                 // past the range: the last row again, never consumed
            __builtin_amdgcn_sched_barrier(0);            // keep the look-ahead loads ahead of the arithmetic
            consume(kA, vA, j0);
            j0 += NW * BK;
            if (j0 >= c1) break;
            request(kA, vA, j0 + NW * BK);
            __builtin_amdgcn_sched_barrier(0);
            consume(kB, vB, j0);
            j0 += NW * BK;
            if (j0 >= c1) break;
        }
    }
    // merge the KPI lane groups of the wave: common maximum, rescale, sum
    float mw = m;
    if (LPK == 8) mw = fmaxf(mw, dpp_f<0x128>(mw));      // lane ^ 8 (rotate the row of 16 by 8)
    mw = fmaxf(mw, __shfl_xor(mw, 16, kWave));
    mw = fmaxf(mw, __shfl_xor(mw, 32, kWave));
    {
        const float r = __builtin_amdgcn_exp2f(m - mw);
        l *= r;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= r;
    }
    if (LPK == 8) l += dpp_f<0x128>(l);
    l += __shfl_xor(l, 16, kWave);
    l += __shfl_xor(l, 32, kWave);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (LPK == 8) acc[e] += dpp_f<0x128>(acc[e]);
        acc[e] += __shfl_xor(acc[e], 16, kWave);
        acc[e] += __shfl_xor(acc[e], 32, kWave);
    }
    if (lane < LPK) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sm_acc[wave][lane * 8 + e] = acc[e];
    }
    if (lane == 0) {
        sm_m[wave] = mw;
        sm_l[wave] = l;
    }
    __syncthreads();
    float M = sm_m[0];                                   // kEmpty only for an empty range
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w]);
    float Lsum = 0.f, A = 0.f;
    if (tid < D) {
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float r = __builtin_amdgcn_exp2f(sm_m[w] - M);              // idle wave: sum and values are zero
            Lsum += sm_l[w] * r;
            A += sm_acc[w][tid] * r;
        }
    }
    if (splits == 1) {
        if (tid < D) a.ctx[bh * D + tid] = (half_t)(Lsum > 0.f ? A / Lsum : 0.f);   // a pair that sees no key: zeros, not 0/0
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
    float Lsum = 0.f, A = 0.f;
    if (splits <= MAXS) {                                // the usual case: everything in one trip to memory
        float mv[MAXS], lv[MAXS], av[MAXS];
#pragma unroll
        for (int u = 0; u < MAXS; ++u) {
            const int s = u < splits ? u : splits - 1;
            mv[u] = ml[s * 2];
            lv[u] = ml[s * 2 + 1];
            av[u] = pa[s * D];
        }
        float M = mv[0];                                 // an empty range reports the finite kEmpty and a zero sum (clamped slots repeat the last range)
#pragma unroll
        for (int u = 1; u < MAXS; ++u) M = fmaxf(M, mv[u]);
#pragma unroll
        for (int u = 0; u < MAXS; ++u) {
            const float sc = u < splits ? exp2f(mv[u] - M) : 0.f;
            Lsum += lv[u] * sc;
            A += av[u] * sc;
        }
        a.ctx[bh * D + dd] = (half_t)(Lsum > 0.f ? A / Lsum : 0.f);
        return;
    }
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, ml[s * 2]);     // an empty range reports the finite kEmpty and a zero sum
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
    a.ctx[bh * D + dd] = (half_t)(Lsum > 0.f ? A / Lsum : 0.f);                 // every range empty: zeros, not 0/0
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
    if (a.d == 128) {
        if (a.read_once) hipLaunchKernelGGL((attn_decode<128, 4, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((attn_decode<128, 4, false>), grid, block, 0, s, a);
    } else {
        if (a.read_once) hipLaunchKernelGGL((attn_decode<64, 4, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((attn_decode<64, 4, false>), grid, block, 0, s, a);
    }
    if (a.splits > 1 && !a.leave_ranges) {
        const int pairs = a.batch * a.heads;
        if (a.d == 128) hipLaunchKernelGGL(attn_decode_combine<128>, dim3((pairs + 1) / 2), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(attn_decode_combine<64>, dim3((pairs + 3) / 4), dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace eet
