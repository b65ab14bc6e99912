// Host-side audit of the LDS hand-over schedules of the two pipelined kernels.
//
// paper_2104_12470_amd/csrc/pipeline.hpp holds, as templates over an executor, the order in which a wave of
// gemm_mfma_dma64 / attn_prefill_wide issues tile loads (global memory -> LDS stage), LDS reads, counter waits and
// barriers.  The kernels instantiate those templates with executors that issue the instructions; this program
// instantiates THE SAME templates with an executor that records them, and checks the record against the rules that
// make the hand-over correct for a workgroup of waves that all run this program and meet only at barriers:
//
//   segment(e) = number of barriers a wave has passed when it issues event e.  Two waves are always inside the same
//   segment or the faster one waits at the barrier that ends it, so "x in every wave happens before y in any wave"
//   holds exactly when segment(x) < segment(y).
//
//   R1  a stage is not overwritten while a read of it can be outstanding: for a read r and a later load g of the same
//       stage, segment(retire r) < segment(issue g).
//   R2  a read that feeds the arithmetic sees a landed tile, landed for every wave: for a consumed read r, the latest
//       earlier load g of its stage carries the tile r expects, and segment(retire g) < segment(issue r).
//   R3  a register buffer is consumed only after the wait that covers its reads, and every wait leaves exactly the
//       stated number of newer requests in flight (counter waits retire oldest first).
//   R4  every (tile, sub-step) is consumed exactly once; reads that are never consumed (the look-ahead past the
//       last tile) may see anything.
//   R5  when the loop is left nothing is in flight: the code after it reuses the stages.
//
// Counters retire in issue order (vmcnt for tile loads, lgkmcnt for LDS reads), which is what the recorder models.
// The same checker must reject planted mistakes (wrong stage, missing barrier, short wait), or it proves nothing.
//
// Usage: pipeline_audit            -> exit status 0 and a line per case, or the first violated rule
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../paper_2104_12470_amd/csrc/pipeline.hpp"

namespace {

struct Load { int ring, stage, tile, issue_pos, issue_seg, retire_pos, retire_seg; };
struct Read { int ring, stage, tile, sub, issue_pos, issue_seg, retire_pos, retire_seg; bool consumed; };

struct Trace {
    std::vector<Load> loads;
    std::vector<Read> reads;
    std::vector<int> loads_in_flight, reads_in_flight;   // indices, oldest first
    int pos = 0, seg = 0;
    std::string error;

    void fail(const std::string& m) { if (error.empty()) error = m; }
    int issue_load(int ring, int stage, int tile) {
        loads.push_back({ring, stage, tile, pos++, seg, -1, -1});
        loads_in_flight.push_back((int)loads.size() - 1);
        return (int)loads.size() - 1;
    }
    int issue_read(int ring, int stage, int tile, int sub) {
        reads.push_back({ring, stage, tile, sub, pos++, seg, -1, -1, false});
        reads_in_flight.push_back((int)reads.size() - 1);
        return (int)reads.size() - 1;
    }
    void retire_loads(size_t keep) {                       // oldest first, `keep` newest stay in flight
        ++pos;
        while (loads_in_flight.size() > keep) {
            Load& g = loads[loads_in_flight.front()];
            g.retire_pos = pos; g.retire_seg = seg;
            loads_in_flight.erase(loads_in_flight.begin());
        }
    }
    void retire_reads(size_t keep) {
        ++pos;
        while (reads_in_flight.size() > keep) {
            Read& r = reads[reads_in_flight.front()];
            r.retire_pos = pos; r.retire_seg = seg;
            reads_in_flight.erase(reads_in_flight.begin());
        }
    }
    void barrier() { ++pos; ++seg; }

    // R1, R2, R5 over the finished record
    void check(const char* what) {
        char buf[256];
        if (!loads_in_flight.empty() || !reads_in_flight.empty()) fail(std::string(what) + ": R5 something is still in flight when the loop is left");
        for (const Read& r : reads) {
            if (r.retire_pos < 0) continue;                // reported by R5
            const Load* latest = nullptr;
            for (const Load& g : loads) {
                if (g.ring != r.ring || g.stage != r.stage) continue;
                if (g.issue_pos > r.issue_pos) {           // R1: overwritten later
                    if (!(r.retire_seg < g.issue_seg)) {
                        snprintf(buf, sizeof buf, "%s: R1 ring %d stage %d: read of tile %d (retired in segment %d) can be outstanding when "
                                 "tile %d is loaded over it (issued in segment %d)", what, r.ring, r.stage, r.tile, r.retire_seg, g.tile, g.issue_seg);
                        fail(buf);
                    }
                } else if (!latest || g.issue_pos > latest->issue_pos) {
                    latest = &g;
                }
            }
            if (!r.consumed) continue;
            if (!latest || latest->tile != r.tile) {
                snprintf(buf, sizeof buf, "%s: R2 ring %d stage %d: a consumed read expects tile %d, the stage holds tile %d", what, r.ring,
                         r.stage, r.tile, latest ? latest->tile : -1);
                fail(buf);
            } else if (latest->retire_pos < 0 || !(latest->retire_seg < r.issue_seg)) {
                snprintf(buf, sizeof buf, "%s: R2 ring %d stage %d tile %d: read in segment %d, but the tile has landed for every wave only "
                         "after segment %d", what, r.ring, r.stage, r.tile, r.issue_seg, latest->retire_seg);
                fail(buf);
            }
        }
    }
};

// ------------------------------------------------------------------------------------------------------------------
// recorder for pipe::gemm_k_loop
// ------------------------------------------------------------------------------------------------------------------
struct GemmRecorder {
    Trace t;
    int nk;
    int buf_read[2] = {-1, -1};                            // latest read group of each register buffer
    int issued = 0;                                        // frag() calls so far
    std::vector<int> consumed;                             // (tile * 4 + sub) per mma, in order
    explicit GemmRecorder(int nk_) : nk(nk_) {}

    void load(int tile, int stage) { t.issue_load(0, stage, tile); }
    template <int L>
    void wait_vmem() { t.retire_loads((size_t)L); }       // the queue retires in issue order: the newest L load() calls stay
    void barrier() { t.barrier(); }
    template <int BUF, int SUB>
    void frag(int stage) {
        // the i-th frag() call feeds the i-th mma(): K tile i / 4, sub-step i % 4 (the call past the last tile feeds none)
        const int idx = issued++;
        if (SUB != idx % 4) t.fail("R4 fragment reads do not walk the sub-steps 0..3 in order");
        if (BUF != (SUB & 1)) t.fail("R3 a sub-step is read into the other sub-steps' buffer");
        if (buf_read[BUF] >= 0 && !t.reads[buf_read[BUF]].consumed && t.reads[buf_read[BUF]].tile < nk)
            t.fail("R3 a register buffer is refilled before its fragments were multiplied");
        buf_read[BUF] = t.issue_read(0, stage, idx / 4, SUB);
    }
    template <int BUF, int SUB, int NEWER>
    void wait_frag() {
        // reads retire in issue order: what stays in flight is the newest frag() call, which must be sub-step NEWER's
        const int n = (int)t.reads_in_flight.size();
        if (NEWER >= 0 && n > 0 && t.reads[t.reads_in_flight[n - 1]].sub != NEWER)
            t.fail("R3 an LDS wait count does not match the order the reads were issued in");
        t.retire_reads(NEWER >= 0 ? 1 : 0);
        if (buf_read[BUF] < 0 || t.reads[buf_read[BUF]].sub != SUB) t.fail("R3 wait_frag names a sub-step that is not in its buffer");
        else if (t.reads[buf_read[BUF]].retire_pos < 0) t.fail("R3 wait_frag leaves the buffer it waits for in flight");
    }
    template <int BUF, int SUB>
    void mma() {
        ++t.pos;
        if (buf_read[BUF] < 0) { t.fail("R3 mma on a buffer that was never read into"); return; }
        Read& r = t.reads[buf_read[BUF]];
        if (r.sub != SUB) t.fail("R3 mma names a sub-step that is not in its buffer");
        if (r.retire_pos < 0) t.fail("R3 mma consumes a buffer whose reads have not been waited for");
        if (r.consumed) t.fail("R4 a fragment is multiplied twice");
        r.consumed = true;
        consumed.push_back(r.tile * 4 + r.sub);
    }
    std::string verdict(const char* what) {
        t.check(what);
        if ((int)consumed.size() != 4 * nk) t.fail(std::string(what) + ": R4 number of multiply steps is not 4 per K tile");
        for (int i = 0; i < (int)consumed.size() && i < 4 * nk; ++i)
            if (consumed[i] != i) t.fail(std::string(what) + ": R4 (tile, sub-step) pairs are not consumed once each, in order");
        for (const Read& r : t.reads)
            if (!r.consumed && r.tile < nk) t.fail(std::string(what) + ": R4 a fragment of a real tile is read and never multiplied");
        return t.error;
    }
};

// ------------------------------------------------------------------------------------------------------------------
// recorder for pipe::gemm_k_loop_interleaved: two fragment buffers, one per k half
// ------------------------------------------------------------------------------------------------------------------
struct HalfStepRecorder {
    Trace t;
    int nk;
    int buf_read[2] = {-1, -1};
    int issued = 0;
    std::vector<int> consumed;
    explicit HalfStepRecorder(int nk_) : nk(nk_) {}
    void load(int tile, int stage) { t.issue_load(0, stage, tile); }
    template <int L>
    void wait_vmem() { t.retire_loads((size_t)L); }
    void barrier() { t.barrier(); }
    template <int H>
    void fetch_half(int stage) {
        const int idx = issued++;
        if (H != idx % 2) t.fail("R4 fragment reads do not alternate between the two k halves");
        if (buf_read[H] >= 0 && !t.reads[buf_read[H]].consumed) t.fail("R3 a fragment buffer is refilled before it was multiplied");
        buf_read[H] = t.issue_read(0, stage, idx / 2, H);
    }
    void wait_fetched() { t.retire_reads(0); }
    template <int H>
    void multiply() {
        ++t.pos;
        if (buf_read[H] < 0) { t.fail("R3 multiply before any fragment was read"); return; }
        Read& r = t.reads[buf_read[H]];
        if (r.retire_pos < 0) t.fail("R3 multiply consumes fragments that have not been waited for");
        if (r.consumed) t.fail("R4 a k half is multiplied twice");
        r.consumed = true;
        consumed.push_back(r.tile * 2 + r.sub);
    }
    // the requests are issued between the multiplies of the phase: in program order after its first multiply, which has
    // checked that its own buffer was waited for; the reads go to the other buffer
    template <int H>
    void mma_half_fetch(int stage) {
        multiply<H>();
        fetch_half<1 - H>(stage);
    }
    template <int H>
    void mma_half_fetch_load(int stage, int tile, int lstage) {
        multiply<H>();
        load(tile, lstage);
        fetch_half<1 - H>(stage);
    }
    std::string verdict(const char* what) {
        t.check(what);
        if ((int)consumed.size() != 2 * nk) t.fail(std::string(what) + ": R4 number of multiply phases is not 2 per K tile");
        for (int i = 0; i < (int)consumed.size() && i < 2 * nk; ++i)
            if (consumed[i] != i) t.fail(std::string(what) + ": R4 k halves are not consumed once each, in order");
        for (const Read& r : t.reads)
            if (!r.consumed && r.tile < nk) t.fail(std::string(what) + ": R4 a fragment of a real tile is read and never multiplied");
        return t.error;
    }
};

// ------------------------------------------------------------------------------------------------------------------
// recorder for pipe::attn_kv_loop (ring 0 = K, ring 1 = V)
// ------------------------------------------------------------------------------------------------------------------
struct AttnRecorder {
    Trace t;
    int nt;
    std::vector<int> k_seen, v_seen;
    explicit AttnRecorder(int nt_) : nt(nt_), k_seen(nt_ + 4, 0), v_seen(nt_ + 4, 0) {}
    void load_k(int tile, int stage) { t.issue_load(0, stage, tile); }
    void load_v(int tile, int stage) { t.issue_load(1, stage, tile); }
    void wait_loads_but_newest_pair() { t.retire_loads(2); }
    void wait_loads_all() { t.retire_loads(0); }
    void barrier() { t.barrier(); }
    void first_scores() {
        const int r = t.issue_read(0, 0, 0, 0);
        t.reads[r].consumed = true;
        ++k_seen[0];
        t.retire_reads(0);                                 // the kernel waits for these reads before it forms the scores
    }
    void step(int jt, int v_stage, int k_stage) {
        const int rv = t.issue_read(1, v_stage, jt, 0);
        t.reads[rv].consumed = true;
        ++v_seen[jt];
        if (jt + 1 < nt) {                                 // the keys of the next tile, when there is one
            const int rk = t.issue_read(0, k_stage, jt + 1, 0);
            t.reads[rk].consumed = true;
            ++k_seen[jt + 1];
        }
    }
    void wait_reads() { t.retire_reads(0); }
    std::string verdict(const char* what) {
        t.check(what);
        for (int j = 0; j < nt; ++j)
            if (k_seen[j] != 1 || v_seen[j] != 1) t.fail(std::string(what) + ": R4 a key or value tile is not consumed exactly once");
        return t.error;
    }
};

// ------------------------------------------------------------------------------------------------------------------
// planted mistakes: copies of the tile kernel's three-stage loop with one thing wrong each
// ------------------------------------------------------------------------------------------------------------------
enum Mistake { kWrongStage, kNoBarrier, kShortWait, kLateLoadWait };

template <class Ops>
void mutant_gemm_loop(Ops& op, int nk, Mistake what) {
    op.load(0, 0);
    if (nk > 1) { op.load(1, 1); op.template wait_vmem<1>(); } else { op.template wait_vmem<0>(); }
    op.barrier();
    op.template frag<0, 0>(0);
    int st = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int st1 = st == 2 ? 0 : st + 1, st2 = st1 == 2 ? 0 : st1 + 1;
        const bool more = kt + 2 < nk;
        if (more) op.load(kt + 2, what == kWrongStage ? st1 : st2);   // kWrongStage: over the tile that is read next
        eet::pipe::gemm_tile_front(op, st);
        op.template wait_frag<0, 2, 3>();
        op.template mma<0, 2>();
        if (what == kShortWait) op.template wait_frag<1, 3, 3>();       // kShortWait: the last reads may still fly at the barrier
        else op.template wait_frag<1, 3, -1>();
        if (what == kLateLoadWait) { if (more) op.template wait_vmem<1>(); }   // kLateLoadWait: the last tiles are never waited for
        else { if (more) op.template wait_vmem<1>(); else op.template wait_vmem<0>(); }
        if (what != kNoBarrier) op.barrier();
        op.template frag<0, 0>(st1);
        op.template mma<1, 3>();
        st = st1;
    }
    op.template wait_frag<0, 0, -1>();
    if (what == kLateLoadWait) op.template wait_vmem<0>();
}

// planted mistake for the one-wave-per-SIMD schedule: the tile after next is requested during the first k half, before
// the barrier that releases the stage it goes to
template <class Ops>
void mutant_interleaved_loop(Ops& op, int nk) {
    op.load(0, 0);
    op.load(nk > 1 ? 1 : 0, 1);
    op.template wait_vmem<1>();
    op.barrier();
    op.template fetch_half<0>(0);
    for (int kt = 0; kt < nk; ++kt) {
        const int st = kt & 1;
        op.wait_fetched();
        op.template mma_half_fetch_load<0>(st, kt + 2 < nk ? kt + 2 : nk - 1, st);
        op.wait_fetched();
        op.template wait_vmem<1>();
        op.barrier();
        op.template mma_half_fetch<1>(st ^ 1);
    }
    op.wait_fetched();
    op.template wait_vmem<0>();
}

int failures = 0;

void expect_ok(const std::string& err, const char* what) {
    if (err.empty()) { printf("ok    %s\n", what); return; }
    printf("FAIL  %s\n      %s\n", what, err.c_str());
    ++failures;
}
void expect_caught(const std::string& err, const char* what) {
    if (!err.empty()) { printf("ok    planted mistake caught: %s\n      (%s)\n", what, err.c_str()); return; }
    printf("FAIL  planted mistake NOT caught: %s\n", what);
    ++failures;
}

}  // namespace

int main() {
    char name[128];
    for (int nk : {1, 2, 3, 4, 5, 6, 7, 16, 64, 192, 768}) {
        {
            GemmRecorder r(nk);
            eet::pipe::gemm_k_loop<2>(r, nk);
            snprintf(name, sizeof name, "tile kernel, two LDS stages, %d K tiles", nk);
            expect_ok(r.verdict(name), name);
        }
        {
            GemmRecorder r(nk);
            eet::pipe::gemm_k_loop<2, true>(r, nk);
            snprintf(name, sizeof name, "tile kernel, two LDS stages with early release, %d K tiles", nk);
            expect_ok(r.verdict(name), name);
        }
        {
            HalfStepRecorder r(nk);
            eet::pipe::gemm_k_loop_interleaved(r, nk);
            snprintf(name, sizeof name, "tile kernel, one wave per SIMD, requests between the multiplies, %d K tiles", nk);
            expect_ok(r.verdict(name), name);
        }
        {
            GemmRecorder r(nk);
            eet::pipe::gemm_k_loop<3>(r, nk);
            snprintf(name, sizeof name, "tile kernel, three LDS stages, %d K tiles", nk);
            expect_ok(r.verdict(name), name);
        }
    }
    for (int nt : {1, 2, 3, 4, 5, 8, 16, 33, 64}) {
        AttnRecorder r(nt);
        eet::pipe::attn_kv_loop(r, nt);
        snprintf(name, sizeof name, "256-row attention, K and V rings of three stages, %d key tiles", nt);
        expect_ok(r.verdict(name), name);
    }
    {   // the tile order visits every tile exactly once, for every grid up to 40 x 40 tiles and a few large ones (all three orders)
        int bad = 0;
        auto check_grid = [&](int tm, int tn) {
            std::vector<int> seen((size_t)tm * tn, 0);
            for (int pid = 0; pid < tm * tn; ++pid) {
                int m = -1, n = -1;
                eet::pipe::tile_of_block(pid, tm, tn, m, n);
                if (m < 0 || m >= tm || n < 0 || n >= tn) { ++bad; continue; }
                ++seen[(size_t)m * tn + n];
            }
            for (int v : seen) bad += v != 1;
        };
        for (int tm = 1; tm <= 40; ++tm)
            for (int tn = 1; tn <= 40; ++tn) check_grid(tm, tn);
        check_grid(96, 192); check_grid(96, 48); check_grid(96, 144); check_grid(13, 16); check_grid(97, 193); check_grid(1, 1000); check_grid(1000, 1);
        check_grid(40, 128); check_grid(8, 512); check_grid(24, 192); check_grid(100, 64); check_grid(16, 48); check_grid(32, 64);   // whole rounds with and without multiples of 16
        expect_ok(bad ? "tile order: some workgroup index maps outside the grid or two map to one tile" : "", "tile order is a bijection");
    }
    const struct { Mistake m; const char* what; } planted[] = {
        {kWrongStage, "next tile loaded over the stage that is read next"},
        {kNoBarrier, "no barrier at the end of a step"},
        {kShortWait, "end of step does not wait for the last fragment reads"},
        {kLateLoadWait, "the last two tiles are not waited for before they are read"},
    };
    for (const auto& p : planted) {
        GemmRecorder r(8);
        mutant_gemm_loop(r, 8, p.m);
        expect_caught(r.verdict(p.what), p.what);
    }
    {
        HalfStepRecorder r(8);
        mutant_interleaved_loop(r, 8);
        const char* what = "one-wave-per-SIMD schedule that requests the tile after next before the stage is released";
        expect_caught(r.verdict(what), what);
    }
    printf(failures ? "pipeline audit: %d FAILED\n" : "pipeline audit: all schedules pass (%d failures)\n", failures);
    return failures ? 1 : 0;
}
