"""Parity of the library's host-side policies (moe_expert_times, moe_greedy_assign, moe_cache_step) with the
scheduling oracle, element by element, on seeded random instances and on the degenerate cases.  Host code only: runs
without a GPU."""
import ctypes as C
import os
import random

import numpy as np
import pytest

from oracle import scheduling as sch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_03495_amd", "libmoe_mi355x.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return C.CDLL(LIB)


def fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def bp(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def lp(a):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def lib_greedy(lib, t_gpu, t_cpu):
    N = len(t_gpu)
    tg, tc = np.asarray(t_gpu, np.float32), np.asarray(t_cpu, np.float32)
    G, Cc = np.zeros(N, np.uint8), np.zeros(N, np.uint8)
    Tg, Tc = C.c_float(0), C.c_float(0)
    assert lib.moe_greedy_assign(N, fp(tg), fp(tc), bp(G), bp(Cc), C.byref(Tg), C.byref(Tc)) == 0
    return Cc.tolist(), G.tolist(), Tc.value, Tg.value


def test_greedy_assign_matches_oracle(lib):
    rng = random.Random(11)
    gpu_tab = np.array([0.0] + [1.0 + 0.0625 * i for i in range(1, 65)], np.float32)     # exactly representable times
    cpu_tab = np.array([0.0] + [0.75 * i for i in range(1, 65)], np.float32)
    for trial in range(400):
        N = rng.choice([1, 2, 8, 60, 64, 128])
        counts = np.array([rng.choice([0, 0, 1, 2, 3, 7, 16, 40, 64, 200]) for _ in range(N)], np.int32)
        cached = np.array([rng.random() < 0.5 for _ in range(N)], np.uint8)
        t_gpu, t_cpu = np.zeros(N, np.float32), np.zeros(N, np.float32)
        assert lib.moe_expert_times(N, ip(counts), bp(cached), C.c_float(2.5), fp(gpu_tab), fp(cpu_tab), 64, fp(t_gpu), fp(t_cpu)) == 0
        og, oc = sch.expert_times(counts.tolist(), cached.tolist(), 2.5, gpu_tab.tolist(), cpu_tab.tolist())
        assert t_gpu.tolist() == og and t_cpu.tolist() == oc
        Cc, G, Tc, Tg = lib_greedy(lib, t_gpu, t_cpu)
        oC, oG, oTc, oTg = sch.greedy_assign(og, oc)
        assert G == oG and Cc == oC
        assert Tg == pytest.approx(oTg, rel=1e-6) and Tc == pytest.approx(oTc, rel=1e-6)


def test_greedy_assign_edge_cases(lib):
    assert lib_greedy(lib, [0.0, 0.0, 0.0], [0.0, 0.0, 0.0])[:2] == ([0, 0, 0], [0, 0, 0])
    assert lib_greedy(lib, [1.0, 1.0, 1.0, 1.0], [1.0, 1.0, 1.0, 1.0])[:2] == ([0, 1, 0, 1], [1, 0, 1, 0])
    assert lib_greedy(lib, [4, 1, 3, 0, 2], [10, 2, 3.5, 0, 8]) == ([0, 1, 1, 0, 0], [1, 0, 0, 0, 1], 5.5, 6.0)
    z = C.c_void_p(0)
    g = np.zeros(4, np.uint8)
    t = np.zeros(4, np.float32)
    assert lib.moe_greedy_assign(0, fp(t), fp(t), bp(g), bp(g), z, z) == -1
    assert lib.moe_greedy_assign(129, fp(t), fp(t), bp(g), bp(g), z, z) == -1
    assert lib.moe_greedy_assign(4, z, fp(t), bp(g), bp(g), z, z) == -1


def test_cache_step_matches_oracle(lib):
    rng = random.Random(5)
    for trial in range(60):
        N = rng.choice([8, 60, 128])
        n = rng.randint(1, N - 1)
        w_size, u_size = rng.choice([1, 2, 4, 8]), rng.choice([0, 1, 2, 8])
        mode = trial % 2                                  # 0: Alg. 2 as printed, 1: the guarded variant
        init = rng.sample(range(N), n)
        oc = sch.WorkloadAwareCache(N, init, w_size, u_size, guarded=bool(mode))
        score = np.zeros(N, np.int64)
        on_gpu = np.zeros(N, np.uint8)
        on_gpu[init] = 1
        step = C.c_int32(0)
        ev, ld = np.full(max(u_size, 1), -1, np.int32), np.full(max(u_size, 1), -1, np.int32)
        nsw = C.c_int32(0)
        hot = rng.sample(range(N), 6)
        for i in range(40):
            w = np.zeros(N, np.int32)
            for e in hot:
                w[e] = rng.randint(0, 6)
            for _ in range(4):
                w[rng.randrange(N)] += rng.randint(0, 3)
            if i % 13 == 12:
                hot = rng.sample(range(N), 6)             # the workload shifts
            swaps = oc.step(w.tolist())
            assert lib.moe_cache_step(N, w_size, u_size, mode, ip(w), lp(score), bp(on_gpu), C.byref(step), ip(ev), ip(ld), C.byref(nsw)) == 0
            assert [(int(ev[j]), int(ld[j])) for j in range(nsw.value)] == swaps
            assert np.nonzero(on_gpu)[0].tolist() == oc.expert_on_gpu
            assert score.tolist() == oc.s and step.value == oc.i % w_size


def test_cache_step_hand_trace_and_errors(lib):
    """The golden window-2 exchange through the C ABI under both modes, and the argument checks."""
    steps = [[0, 1, 0, 0, 3, 0, 2, 0], [1, 0, 0, 0, 2, 0, 2, 1], [0, 0, 1, 0, 3, 1, 1, 0], [0, 1, 0, 0, 2, 0, 3, 0]] + [[0, 0, 0, 0, 2, 0, 2, 0]] * 4
    for mode, want2, after2 in ((0, [(1, 0), (2, 3)], [0, 3, 4, 6]), (1, [], [1, 2, 4, 6])):
        score, on_gpu = np.zeros(8, np.int64), np.array([1, 1, 1, 1, 0, 0, 0, 0], np.uint8)
        step, nsw = C.c_int32(0), C.c_int32(0)
        ev, ld = np.full(2, -1, np.int32), np.full(2, -1, np.int32)
        got = []
        for w in steps:
            wa = np.array(w, np.int32)
            assert lib.moe_cache_step(8, 4, 2, mode, ip(wa), lp(score), bp(on_gpu), C.byref(step), ip(ev), ip(ld), C.byref(nsw)) == 0
            got.append([(int(ev[j]), int(ld[j])) for j in range(nsw.value)])
        assert got[3] == [(3, 4), (0, 6)] and got[7] == want2
        assert [g for i, g in enumerate(got) if i not in (3, 7)] == [[]] * 6
        assert np.nonzero(on_gpu)[0].tolist() == after2
    wa, score, on_gpu = np.zeros(8, np.int32), np.zeros(8, np.int64), np.zeros(8, np.uint8)
    step, nsw = C.c_int32(0), C.c_int32(0)
    ev = np.zeros(2, np.int32)
    args = (ip(wa), lp(score), bp(on_gpu), C.byref(step), ip(ev), ip(ev), C.byref(nsw))
    assert lib.moe_cache_step(8, 4, 2, 2, *args) == -1            # unknown mode
    assert lib.moe_cache_step(8, 0, 2, 0, *args) == -1
    assert lib.moe_cache_step(129, 4, 2, 0, *args) == -1
