// The LDS hand-over schedules of the two pipelined kernels, written once.
//
// gemm_mfma_dma64 (gemm.hip) and attn_prefill_wide (attention.hip) move operand tiles from global memory
// straight into rings of LDS stages while other waves still read earlier tiles out of the same ring.  What
// makes that correct is only the ORDER in which a wave issues tile loads, fragment reads, counter waits and
// barriers.  That order lives here, as templates over an executor:
//   * in the kernels the executor issues the instructions (its methods are forced inline: the generated code
//     is the same as if the loop were written out in the kernel);
//   * in tests/pipeline_audit.cpp, a host program, the executor records them, and a checker replays the
//     record for all waves of a workgroup and asserts that no stage is overwritten while a read of it can be
//     outstanding, that no fragment is consumed before its tile has landed for every wave, that every
//     (K tile, K sub-step) is multiplied exactly once, and that nothing is in flight when the loop is left.
// This header is plain C++ (no HIP types), so the host program includes the very text the kernels compile.
#pragma once

#if defined(__HIPCC__) || defined(__HIP__)
#define EET_PIPE_FN __host__ __device__ __forceinline__
#else
#define EET_PIPE_FN inline
#endif

namespace eet {
namespace pipe {

// ---------------------------------------------------------------------------------------------------------
// Tile order of the MFMA tile kernel.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): workgroup
// pid runs on XCD pid % 8 and is the (pid / 8)-th there; with one workgroup per CU (the 256 x 256 tiles) the 32 CUs of
// an XCD work on 32 consecutive workgroups of theirs at a time.  Every workgroup index in [0, tiles_m * tiles_n) maps to
// a different tile (checked on the host for all small grids and the large ones in use).
//   * Whole rounds of 256 tiles, from two rounds on, both tile counts multiples of 16: round r is one super-block of
//     16 x 16 tiles (row-major over the super-blocks, so consecutive rounds keep their 16 row tiles), of which XCD x takes
//     the 8 x 4 block at (x / 4, x % 4).  The chip then reads 32 operand panels per round instead of the 96 of eight
//     unrelated blocks, and an XCD shares its 12 with its neighbours through the memory-side cache (rows x N x K:
//     24576 x 49152 x 12288 23.9 -> 21.35 ms, 24576 x 36864 x 12288 17.67 -> 16.05, 24576 x 12288 x 12288 6.00 -> 5.58,
//     24576 x 12288 x 49152 23.3 -> 22.5, 8192 x 16384 x 12288 2.51 -> 2.43; nothing lost at 3 or 4 rounds).
//   * Whole rounds, 16 rounds or more, other tile counts: block k of 32 consecutive positions of the sequence below goes
//     to XCD k % 8, so the XCDs work side by side on one group of 8 row tiles (about two thirds of the gain above on the
//     same shapes; with few rounds it loses: 4096 x 12288 x 12288 0.92 -> 0.97 ms).
//   * Otherwise XCD x is given a contiguous range of a tile sequence in which any 32 consecutive tiles form a block of
//     8 row-tiles x 4 column-tiles: 12 operand panels are shared by 32 tiles.
// ---------------------------------------------------------------------------------------------------------
EET_PIPE_FN void tile_of_block(int pid, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    constexpr int GM = 8;
    const int nb = tiles_m * tiles_n;
    const int xcd = pid & 7, local = pid >> 3;
    const bool whole_rounds = (nb & 255) == 0;
    if (whole_rounds && nb >= 512 && (tiles_m & 15) == 0 && (tiles_n & 15) == 0) {
        const int sb = local >> 5, w = local & 31, sbn_count = tiles_n >> 4;
        const int sbm = sb / sbn_count, sbn = sb - sbm * sbn_count;
        tile_m = sbm * 16 + (xcd >> 2) * 8 + (w & 7);
        tile_n = sbn * 16 + (xcd & 3) * 4 + (w >> 3);
        return;
    }
    const int q = nb >> 3, rem = nb & 7;
    int t = xcd * q + (xcd < rem ? xcd : rem) + local;         // position in the sequence
    if (whole_rounds && nb >= 4096) t = ((local >> 5) * 8 + xcd) * 32 + (local & 31);
    const int per_group = GM * tiles_n;
    const int grp = t / per_group, in_grp = t - grp * per_group;
    const int gm0 = grp * GM;
    const int gsz = tiles_m - gm0 < GM ? tiles_m - gm0 : GM;    // last group may be shorter
    tile_n = in_grp / gsz;
    tile_m = gm0 + in_grp - tile_n * gsz;
}

// ---------------------------------------------------------------------------------------------------------
// K loop of the MFMA tile kernel: K tiles of 64 columns through NS LDS stages (tile t in stage t % NS), four
// sub-steps per tile, fragments double-buffered in registers (buffer = sub-step % 2).
//
// Executor interface (SUB = sub-step 0..3 of a tile, BUF = SUB % 2 its register buffer, stage = ring slot):
//   load(tile, stage)            issue this wave's global->LDS loads of K tile `tile`           (vector-memory counter)
//   wait_vmem<L>()               the loads of this wave have landed, except those of the newest L load() calls (the
//                                vector-memory queue retires in issue order)
//   barrier()                    workgroup barrier
//   frag<BUF, SUB>(stage)        issue the LDS reads of sub-step SUB of the tile in `stage` into buffer BUF
//   wait_frag<BUF, SUB, NEWER>() the reads of sub-step SUB have landed; those of sub-step NEWER, issued after them, may
//                                still fly (NEWER = -1: none: every read of this wave has landed)
//   mma<BUF, SUB>()              multiply-accumulate sub-step SUB from buffer BUF
// ---------------------------------------------------------------------------------------------------------
// the three sub-steps in the middle of a tile, common to every schedule: on entry the reads of sub-step 0 are in flight
template <class Ops>
EET_PIPE_FN void gemm_tile_front(Ops& op, int st) {
    op.template frag<1, 1>(st);
    op.template wait_frag<0, 0, 1>();
    op.template mma<0, 0>();
    op.template frag<0, 2>(st);
    op.template wait_frag<1, 1, 2>();
    op.template mma<1, 1>();
    op.template frag<1, 3>(st);
}

template <int NS, bool EARLY = false, class Ops = void>
EET_PIPE_FN void gemm_k_loop(Ops& op, int nk) {
    static_assert(NS == 2 || NS == 3, "LDS stages");
    static_assert(!EARLY || NS == 2, "early release: two-stage schedule only");
    if (NS == 2 && EARLY) {
        // two stages, early release: the reads of a tile's last sub-step are issued after the multiplies of its second,
        // and the barrier that hands the stage over sits before the multiplies of the last two sub-steps; the request of
        // tile kt+2 follows the barrier at once, while the fetch of tile kt+1 is still completing
        op.load(0, 0);
        op.template wait_vmem<0>();
        op.barrier();
        if (nk > 1) op.load(1, 1);
        op.template frag<0, 0>(0);
        for (int kt = 0; kt < nk; ++kt) {
            const int st = kt & 1;
            gemm_tile_front(op, st);
            op.template wait_frag<1, 3, -1>();    // every read of stage st has landed (sub-steps 2 and 3 sit in the buffers)
            op.template wait_frag<0, 2, -1>();
            op.template wait_vmem<0>();        // this wave's part of tile kt+1 has landed
            op.barrier();                         // ... and everybody else's; stage st is free
            if (kt + 2 < nk) op.load(kt + 2, st);
            op.template mma<0, 2>();
            op.template frag<0, 0>(st ^ 1);       // (past the last tile: stale data, never multiplied)
            op.template mma<1, 3>();
        }
    } else if (NS == 2) {
        // two stages: tile kt+1 is requested at the start of step kt into the stage that step kt-1 read and that the
        // barrier at its end released; the end of step kt waits for it
        op.load(0, 0);
        op.template wait_vmem<0>();
        op.barrier();
        op.template frag<0, 0>(0);
        for (int kt = 0; kt < nk; ++kt) {
            const int st = kt & 1;
            if (kt + 1 < nk) op.load(kt + 1, st ^ 1);
            gemm_tile_front(op, st);
            op.template wait_frag<0, 2, 3>();
            op.template mma<0, 2>();
            op.template wait_frag<1, 3, -1>();    // all of this wave's reads of stage st are done
            op.template wait_vmem<0>();           // this wave's part of tile kt+1 has landed
            op.barrier();                         // ... and everybody else's; stage st is free
            op.template frag<0, 0>(st ^ 1);       // (past the last tile: stale data, never multiplied)
            op.template mma<1, 3>();
        }
    } else {
        // ring of three stages: tile kt+2 is requested at the start of step kt, into the stage that step kt-1 read and
        // the barrier at its end released; at the end of step kt only that newest request may still be in flight
        op.load(0, 0);
        if (nk > 1) {
            op.load(1, 1);
            op.template wait_vmem<1>();
        } else {
            op.template wait_vmem<0>();
        }
        op.barrier();                             // nothing but the loads above has touched LDS so far
        op.template frag<0, 0>(0);
        int st = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const int st1 = st == 2 ? 0 : st + 1, st2 = st1 == 2 ? 0 : st1 + 1;
            const bool more = kt + 2 < nk;
            if (more) op.load(kt + 2, st2);
            gemm_tile_front(op, st);
            op.template wait_frag<0, 2, 3>();
            op.template mma<0, 2>();
            op.template wait_frag<1, 3, -1>();    // all of this wave's reads of stage st are done
            if (more) op.template wait_vmem<1>(); else op.template wait_vmem<0>();   // this wave's part of tile kt+1 has landed
            op.barrier();                         // ... and everybody else's; stage st is free
            op.template frag<0, 0>(st1);          // (past the last tile: stale data, never multiplied)
            op.template mma<1, 3>();
            st = st1;
        }
    }
    op.template wait_frag<0, 0, -1>();            // the stale reads too: the epilogue reuses the stages
}

// ---------------------------------------------------------------------------------------------------------
// K loop of the MFMA tile kernel for one wave per SIMD, two LDS stages.  Nothing else runs on the SIMD while a wave
// waits, and the LDS of the CU is busy most of the time (fragment reads of four waves plus the arriving tiles), so
// every request is issued between the multiplies of an earlier phase, spread evenly over them: a burst of LDS reads
// stalls the wave's instruction stream, and the multiplies behind it, until the LDS queue has room.
//
// A K tile is two phases, one per k half; the fragments of a whole k half have two register buffers (buffer = k half).
// While k half 0 of tile kt is multiplied the reads of its k half 1 are issued.  After them every read of the stage
// has been issued: the wave waits for them and for its part of tile kt+1, and the barrier hands the stage over with
// half of the tile's multiplies still to come.  While k half 1 is multiplied the loads of tile kt+2 go into the stage
// just released and the reads of k half 0 of tile kt+1 are issued.  The loads past the last tile repeat the last tile
// (the number of loads per step, and with it every wait count, stays fixed; nothing reads them).
//
// Executor interface: load(tile, stage), wait_vmem<L>(), barrier() as for gemm_k_loop, and
//   fetch_half<H>(stage)                        issue the LDS reads of k half H of the tile in `stage` into buffer H
//   wait_fetched()                              every LDS read of this wave has landed
//   mma_half_fetch<H>(stage)                    multiply k half H out of buffer H; between the multiplies issue the reads
//                                               of k half 1-H of `stage` into the other buffer
//   mma_half_fetch_load<H>(stage, tile, lstage) the same, and issue the loads of K tile `tile` into stage `lstage`
// ---------------------------------------------------------------------------------------------------------
template <class Ops>
EET_PIPE_FN void gemm_k_loop_interleaved(Ops& op, int nk) {
    op.load(0, 0);
    op.load(nk > 1 ? 1 : 0, 1);
    op.template wait_vmem<1>();                   // tile 0 of this wave has landed ...
    op.barrier();                                 // ... and everybody else's
    op.template fetch_half<0>(0);
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        op.wait_fetched();
        op.template mma_half_fetch<0>(st);
        op.wait_fetched();                          // every read of stage st has landed
        op.template wait_vmem<0>();               // this wave's part of tile kt+1 has landed
        op.barrier();                             // ... and everybody else's; stage st is free
        op.template mma_half_fetch_load<1>(st ^ 1, kt + 2 < nk ? kt + 2 : nk - 1, st);   // (reads past the last tile: stale, never multiplied)
    }
    op.wait_fetched();                              // the stale reads and the repeated loads too: the epilogue reuses the stages
    op.template wait_vmem<0>();
}

// ---------------------------------------------------------------------------------------------------------
// Key-tile loop of the 256-row prefill attention: K and V tiles of 64 keys through two rings of three stages
// (tile t in stage t % 3 of its ring).  During step jt the waves read V(jt) and K(jt+1) -- the scores of tile
// jt were formed during step jt-1 -- while K(jt+2), V(jt+1) (requested during step jt-1) and K(jt+3), V(jt+2)
// (requested at the start of this step, into the stages step jt-1 was reading) are in flight.  Requests past
// the last tile are still issued (the kernel clamps their rows): the number of loads per step, and with it
// every wait count, stays fixed.
//
// Executor interface:
//   load_k(tile, stage), load_v(tile, stage)   issue this wave's global->LDS loads of a key / value tile
//   wait_loads_but_newest_pair()               every load except those of the newest load_k + load_v pair has landed
//   wait_loads_all()
//   barrier()
//   first_scores()                             reads K(0) out of K stage 0 and waits for them (scores of tile 0)
//   step(jt, v_stage, k_stage)                 reads V(jt) from v_stage and K(jt+1) from k_stage, multiplies
//   wait_reads()                               every LDS read of this wave has landed
// ---------------------------------------------------------------------------------------------------------
template <class Ops>
EET_PIPE_FN void attn_kv_loop(Ops& op, int nt) {
    op.load_k(0, 0);
    op.load_k(1, 1);
    op.load_v(0, 0);
    op.load_k(2, 2);
    op.load_v(1, 1);
    op.wait_loads_but_newest_pair();              // K(0), K(1), V(0) of this wave have landed ...
    op.barrier();                                 // ... and everybody else's
    op.first_scores();
    op.wait_reads();
    op.barrier();                                 // step 0 refills the stage of K(0)
    int s0 = 0;                                   // stage of tile jt
    for (int jt = 0; jt < nt; ++jt) {
        const int s1 = s0 == 2 ? 0 : s0 + 1, s2 = s0 == 0 ? 2 : s0 - 1;
        op.load_k(jt + 3, s0);                    // K(jt) was last read during step jt-1
        op.load_v(jt + 2, s2);                    // V(jt-1) was last read during step jt-1
        op.step(jt, s0, s1);
        op.wait_reads();                          // this wave is done reading the stages of this step
        op.wait_loads_but_newest_pair();          // K(jt+2), V(jt+1) of this wave have landed ...
        op.barrier();                             // ... and everybody else's
        s0 = s1;
    }
    op.wait_loads_all();                          // no load may still be writing LDS when the workgroup ends
}

}  // namespace pipe
}  // namespace eet
