"""Buffer manager of Section 3.2: pins of the oracle (CPU), and the library's manager against the oracle
through the C ABI (CPU: the manager is host logic over an arena it never dereferences)."""
import ctypes as C
import os

import pytest

from oracle import buffer_manager as obm
from oracle import eet_oracle as orc
from paper_2104_12470_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "buffer_manager_scenario.txt")


def scenario():
    """-> (events, expected footprint); events: ("req", module, bytes, number, offset, how) / ("rel", number)"""
    ev, foot = [], None
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if not t:
            continue
        if t[0] == "req":
            ev.append(("req", int(t[1]), int(t[2]), int(t[4]), int(t[5]), t[6]))
        elif t[0] == "rel":
            ev.append(("rel", int(t[1])))
        elif t[0] == "footprint":
            foot = int(t[1])
    return ev, foot


def run_scenario(mgr):
    """Replays the golden scenario; returns the list of mismatches against the hand-worked decisions."""
    ev, foot = scenario()
    offset_of, bad = {}, []
    for e in ev:
        if e[0] == "req":
            _, module, nbytes, number, offset, how = e
            got = mgr.request(nbytes, module)
            if got != (offset, how):
                bad.append((e, got))
            offset_of[number] = got[0]
        else:
            mgr.release(offset_of[e[1]])
    if mgr.footprint != foot:
        bad.append(("footprint", mgr.footprint))
    return bad


def test_oracle_follows_the_hand_worked_scenario():
    assert run_scenario(obm.BufferManagerOracle(1 << 20)) == []


class _FirstFitAnyModule(obm.BufferManagerOracle):          # planted mistake: R1 dropped
    def request(self, nbytes, module):
        size = self._round(nbytes)
        for b in self.buffers:
            if b.idle and size <= b.size:
                b.idle, b.module = False, module
                return b.offset, "same_size" if size == b.size else "larger"
        return super().request(nbytes, module)


class _ExactOnly(obm.BufferManagerOracle):                   # planted mistake: R2 dropped
    def request(self, nbytes, module):
        size = self._round(nbytes)
        for b in self.buffers:
            if b.idle and size == b.size:
                b.idle, b.module = False, module
                return b.offset, "same_size"
        saved = [(b, b.idle) for b in self.buffers]
        for b in self.buffers:
            b.idle = False
        try:
            return super().request(nbytes, module)
        finally:
            for b, idle in saved:
                b.idle = idle


class _BestFit(obm.BufferManagerOracle):                     # planted mistake: best fit instead of first fit
    def request(self, nbytes, module):
        size = self._round(nbytes)
        ok = [b for b in self.buffers if b.idle and ((b.module == module and b.size == size) or
                                                     (b.module != module and size <= b.size))]
        if ok:
            b = min(ok, key=lambda x: x.size)
            how = "same_size" if b.size == size else "larger"
            b.idle, b.module = False, module
            return b.offset, how
        return super().request(nbytes, module)


@pytest.mark.parametrize("wrong", [_FirstFitAnyModule, _ExactOnly, _BestFit])
def test_scenario_catches_planted_mistakes(wrong):
    assert run_scenario(wrong(1 << 20)) != []


def replay(mgr, trace):
    off = {}
    for e in trace:
        if e[0] == "req":
            off[e[1]] = mgr.request(e[2], e[3])[0]
        else:
            mgr.release(off.pop(e[1]))
    return off


@pytest.mark.parametrize("b,p,h,n", [(4, 1024, 1600, 25), (8, 512, 1024, 16), (2, 4096, 2048, 16)])
def test_unfused_layer_reproduces_the_total_of_section_3_2(b, p, h, n):
    """With n*p >= 4h the feed-forward intermediate fits the idle score buffer (rule R2), the context buffers
    reuse q and k (rule R1), and the total is the paper's b*p*(6h + n*p) elements."""
    assert n * p >= 4 * h
    mgr = obm.BufferManagerOracle(1 << 40)
    trace = wl.unfused_layer_buffer_trace(b, p, h, n, 4 * h)
    replay(mgr, trace)
    assert mgr.footprint == 2 * orc.buffer_elements(b, p, h, n)
    assert mgr.counts["created"] == 5 and mgr.counts["same_size"] == 2 and mgr.counts["larger"] == 1
    before = mgr.footprint
    for _ in range(3):                                  # the next layers, the next calls: nothing new (Section 3.1)
        replay(mgr, trace)
    assert mgr.footprint == before and mgr.counts["created"] == 5


def test_short_prompts_need_a_buffer_of_their_own_for_the_feed_forward():
    b, p, h, n = 4, 64, 768, 12                          # n*p < 4h: no idle buffer is large enough
    mgr = obm.BufferManagerOracle(1 << 40)
    replay(mgr, wl.unfused_layer_buffer_trace(b, p, h, n, 4 * h))
    assert mgr.footprint == 2 * (orc.buffer_elements(b, p, h, n) + b * p * 4 * h)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_live_buffers_never_overlap(seed):
    mgr = obm.BufferManagerOracle(1 << 30)
    off = {}
    for e in wl.random_buffer_trace(seed, 400):
        if e[0] == "req":
            off[e[1]] = mgr.request(e[2], e[3])[0]
        else:
            mgr.release(off.pop(e[1]))
        spans = sorted(mgr.live())
        assert all(a[0] + a[1] <= b_[0] for a, b_ in zip(spans, spans[1:]))
        assert len(spans) == len(off)
        assert mgr.footprint == sum(b_.size for b_ in mgr.buffers) <= mgr.arena_bytes


def test_oracle_errors():
    mgr = obm.BufferManagerOracle(1024)
    with pytest.raises(obm.BufferError):
        mgr.request(0, 0)
    a, _ = mgr.request(700, 0)                           # 768 of 1024 bytes
    with pytest.raises(obm.BufferError):
        mgr.request(512, 0)                              # does not fit; nothing changes
    assert mgr.footprint == 768 and len(mgr.buffers) == 1
    mgr.release(a)
    with pytest.raises(obm.BufferError):
        mgr.release(a)
    with pytest.raises(obm.BufferError):
        mgr.release(12345)


# ---- the library's manager against the oracle, through the C ABI (host logic: runs without a GPU) ----------
ARENA = 0x7F0000000000                      # an address, never dereferenced by the manager


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2104_12470_amd.build import build_library
        build_library(verbose=False)
    binding.lib()
    return binding


class _LibManager:
    """The library's manager behind the oracle's interface (offsets instead of pointers)."""

    def __init__(self, eet, arena_bytes):
        self.eet, self.h = eet, eet.eet_bufmgr_create(ARENA, arena_bytes)

    def request(self, nbytes, module):
        before = self.eet.eet_bufmgr_query(self.h)
        p = self.eet.eet_bufmgr_request(self.h, nbytes, module)
        after = self.eet.eet_bufmgr_query(self.h)
        how = ("created" if after.created > before.created else
               "larger" if after.reused_larger > before.reused_larger else "same_size")
        return p - ARENA, how

    def release(self, offset):
        self.eet.eet_bufmgr_release(self.h, ARENA + offset)

    @property
    def footprint(self):
        return self.eet.eet_bufmgr_query(self.h).footprint_bytes

    def close(self):
        self.eet.eet_bufmgr_destroy(self.h)


def test_library_follows_the_hand_worked_scenario(eet):
    m = _LibManager(eet, 1 << 20)
    assert run_scenario(m) == []
    m.close()


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_library_equals_oracle_on_random_traces(eet, seed):
    arena = 48 * 256 if seed == 14 else 1 << 24          # seed 14: a small arena, so that some requests fail
    lib_m, ora = _LibManager(eet, arena), obm.BufferManagerOracle(arena)
    off, failures = {}, 0
    for e in wl.random_buffer_trace(seed, 600):
        if e[0] == "req":
            try:
                want = ora.request(e[2], e[3])
            except obm.BufferError:
                with pytest.raises(eet.EETError) as err:
                    lib_m.request(e[2], e[3])
                assert err.value.code == eet.EET_ERR_CAPACITY
                failures += 1
                continue
            assert lib_m.request(e[2], e[3]) == want          # same buffer, same reason: exact integers
            off[e[1]] = want[0]
        elif e[1] in off:
            ora.release(off[e[1]])
            lib_m.release(off.pop(e[1]))
        st = eet.eet_bufmgr_query(lib_m.h)
        assert st.footprint_bytes == ora.footprint and st.buffers == len(ora.buffers)
        assert st.idle == sum(b.idle for b in ora.buffers)
        assert (st.requests, st.reused_same_size, st.reused_larger, st.created) == \
            (ora.counts["requests"], ora.counts["same_size"], ora.counts["larger"], ora.counts["created"])
    assert (failures > 0) == (seed == 14)
    lib_m.close()


def test_library_unfused_layer_total(eet):
    b, p, h, n = 4, 1024, 1600, 25
    m = _LibManager(eet, 1 << 40)
    for _ in range(3):
        replay(m, wl.unfused_layer_buffer_trace(b, p, h, n, 4 * h))
    assert m.footprint == 2 * orc.buffer_elements(b, p, h, n)          # Section 3.2: b*p*(6h + n*p) elements, fp16
    m.close()


def test_library_errors(eet):
    L = eet.lib()
    h = C.c_void_p()
    assert L.eet_bufmgr_create(None, 1024, C.byref(h)) == eet.EET_ERR_INVALID_ARG
    assert L.eet_bufmgr_create(ARENA + 8, 1024, C.byref(h)) == eet.EET_ERR_INVALID_ARG       # misaligned arena
    assert L.eet_bufmgr_create(ARENA, 0, C.byref(h)) == eet.EET_ERR_INVALID_ARG
    assert L.eet_bufmgr_create(ARENA, 1024, C.byref(h)) == eet.EET_OK
    p = C.c_void_p()
    assert L.eet_bufmgr_request(h, 0, 0, C.byref(p)) == eet.EET_ERR_INVALID_ARG
    assert L.eet_bufmgr_request(h, 700, 0, C.byref(p)) == eet.EET_OK and p.value == ARENA
    q = C.c_void_p()
    assert L.eet_bufmgr_request(h, 512, 0, C.byref(q)) == eet.EET_ERR_CAPACITY and q.value is None
    assert b"do not fit" in L.eet_last_error()
    assert L.eet_bufmgr_release(h, ARENA + 256) == eet.EET_ERR_INVALID_ARG
    assert L.eet_bufmgr_release(h, p) == eet.EET_OK
    assert L.eet_bufmgr_release(h, p) == eet.EET_ERR_STATE
    st = eet.eet_bufmgr_query(h)
    assert (st.footprint_bytes, st.buffers, st.idle, st.created) == (768, 1, 1, 1)
    assert L.eet_bufmgr_destroy(h) == eet.EET_OK
