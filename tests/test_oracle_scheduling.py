"""Pins of the scheduling oracle (Alg. 1 and Alg. 2): hand traces, exhaustive optimum, closed forms, invariants."""
import os
import random

import pytest

from oracle import scheduling as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scheduling_hand_traces.txt")


def golden(kind):
    for line in open(GOLDEN):
        line = line.strip()
        if line.startswith(kind + " "):
            yield [p.strip() for p in line[len(kind):].split("|")]


def test_greedy_hand_traces():
    n = 0
    for tg, tc, G, C, tot in golden("greedy"):
        t_gpu, t_cpu = [float(x) for x in tg.split()], [float(x) for x in tc.split()]
        c, g, T_cpu, T_gpu = sch.greedy_assign(t_gpu, t_cpu)
        assert g == [int(x) for x in G.split()] and c == [int(x) for x in C.split()]
        assert [T_gpu, T_cpu] == [float(x) for x in tot.split()]
        n += 1
    assert n == 2


def test_greedy_invariants_and_exhaustive_optimum():
    rng = random.Random(7)
    ratios = []
    for trial in range(300):
        N = rng.randint(1, 10)
        w = [rng.choice([0, 0, 1, 2, 5, 9, 16]) for _ in range(N)]
        t_gpu, t_cpu = sch.expert_times(w, None, 3.0, [0.0] + [1.0 + 0.05 * i for i in range(1, 17)],
                                        [0.0] + [0.9 * i for i in range(1, 17)])
        C, G, T_cpu, T_gpu = sch.greedy_assign(t_gpu, t_cpu)
        for i in range(N):
            assert C[i] + G[i] <= 1                                      # mutual exclusion
            assert (C[i] + G[i] == 0) == (w[i] == 0)                     # exactly the activated experts are assigned
        assert sum(C) + sum(G) == sum(1 for x in w if x > 0)             # activation constraint
        assert abs(T_gpu - sum(t for t, g in zip(t_gpu, G) if g)) < 1e-9
        assert abs(T_cpu - sum(t for t, c in zip(t_cpu, C) if c)) < 1e-9
        opt = sch.optimal_assign(t_gpu, t_cpu)
        got = max(T_gpu, T_cpu)
        assert got >= opt - 1e-9                                         # nothing beats the exhaustive optimum
        if got > 0:
            ratios.append(opt / got)
    assert sum(ratios) / len(ratios) > 0.85                             # a heuristic close to optimal (the paper quotes up to 92 %)


def test_greedy_special_cases():
    # one activated expert goes where it is faster, the GPU on a tie
    assert sch.greedy_assign([2.0], [3.0])[1] == [1]
    assert sch.greedy_assign([3.0], [2.0])[0] == [1]
    assert sch.greedy_assign([2.0], [2.0])[1] == [1]
    # nothing activated: nothing assigned
    assert sch.greedy_assign([0.0, 0.0], [0.0, 0.0])[:2] == ([0, 0], [0, 0])
    # a GPU that costs nothing takes everything
    C, G, _, _ = sch.greedy_assign([1e-9] * 6, [5.0] * 6)
    assert G == [1] * 6 and C == [0] * 6
    # the expert with the largest time difference is decided first
    C, G, _, _ = sch.greedy_assign([1.0, 1.0, 1.0], [1.5, 9.0, 1.2])
    assert G[1] == 1


def test_expert_times_cost_model():
    gpu = [0.0, 1.0, 1.1, 1.2]
    cpu = [0.0, 2.0, 4.0, 6.0]
    t_gpu, t_cpu = sch.expert_times([0, 1, 3, 7], [0, 0, 1, 0], 5.0, gpu, cpu)
    assert t_gpu == [0.0, 5.0, 1.2, 5.0]          # transfer dominates unless cached; not activated -> 0
    assert t_cpu == [0.0, 2.0, 6.0, 6.0]          # tables clamp at their last entry


def test_cache_hand_trace():
    (cfg, init, steps, swaps1, after1, swaps2), = list(golden("cache"))
    N, w_size, u_size = (int(x) for x in cfg.split())
    cache = sch.WorkloadAwareCache(N, [int(x) for x in init.split()], w_size, u_size)
    wl_steps = [[int(x) for x in s.split()] for s in steps.split(";")]
    out = [cache.step(w) for w in wl_steps[:4]]
    assert out[:3] == [[], [], []]
    assert out[3] == [tuple(int(x) for x in p.split(">")) for p in swaps1.split()]
    assert cache.expert_on_gpu == [int(x) for x in after1.split()]
    assert cache.s == [0] * N
    out2 = [cache.step(w) for w in wl_steps[4:]]
    assert swaps2 == "none" and out2 == [[], [], [], []]
    assert cache.expert_on_gpu == [int(x) for x in after1.split()]


def test_cache_invariants_and_convergence():
    rng = random.Random(3)
    N, n = 16, 6
    cache = sch.WorkloadAwareCache(N, list(range(n)), w_size=4, u_size=3)
    hot = [9, 11, 12, 13, 14, 15]
    for i in range(64):
        w = [0] * N
        for e in hot:
            w[e] = rng.randint(2, 5)
        w[rng.randrange(N)] += 1
        swaps = cache.step(w)
        assert len(cache.expert_on_gpu) == n and len(set(cache.expert_on_gpu) | set(cache.expert_on_cpu)) == N
        assert len(swaps) <= 3 and (len(swaps) == 0 or (i + 1) % 4 == 0)
    assert set(cache.expert_on_gpu) == set(hot)                         # the persistently hot experts end up cached
    # u_size = 0 never swaps; w_size = 1 swaps after every token
    c0 = sch.WorkloadAwareCache(4, [0, 1], 2, 0)
    assert [c0.step([0, 0, 5, 5]) for _ in range(4)] == [[], [], [], []]
    c1 = sch.WorkloadAwareCache(4, [0, 1], 1, 1)
    assert c1.step([0, 0, 5, 4]) == [(0, 2)]
