"""CPU oracle of the paper's two host-side policies -- TEST INFRASTRUCTURE ONLY.

Plain Python, written from Alg. 1 (Greedy Assignment Strategy) and Alg. 2 (Workload-Aware Cache Replacement) and
the text around them, in the paper's notation.  Shares nothing with the library's implementation.

Readings where the paper is silent or at odds with itself:
  * Alg. 1 sorts by |t_gpu - t_cpu| descending; equal differences keep ascending expert index (stable sort).
  * Alg. 2's second TopK is printed like the first, but the text says the experts with the LOWEST scores on the GPU
    are evicted; the text is followed.
  * Alg. 2 tests `i mod w_size == 0`, which would fire on the very first token; the text says "after processing a
    window of w_size tokens", so the replacement happens when (i + 1) mod w_size == 0.
  * Equal scores: lower expert index first, on both sides.  When fewer than u_size experts are on one side, as many
    as both sides have are exchanged.

Alg. 2 and the paragraph before it exchange u_size experts at every window end, whatever their scores: that is what
`WorkloadAwareCache` does by default.  `guarded=True` selects a variant that is NOT the paper's: a pair is exchanged
only while the incoming expert's score is larger than the outgoing one's.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def expert_times(counts: Sequence[int], cached, trans_time: float, gpu_compute: Sequence[float],
                 cpu_compute: Sequence[float]) -> Tuple[List[float], List[float]]:
    """t_gpu(w) = max(Trans(w), compute(w)) with Trans(w) = 0 for w = 0 or a cached expert, else trans_time;
    t_cpu(w) from its table; both 0 for experts that are not activated (Section "Greedy Assignment Strategy")."""
    t_gpu, t_cpu = [], []
    wmax = len(gpu_compute) - 1
    for e, w in enumerate(counts):
        if w == 0:
            t_gpu.append(0.0)
            t_cpu.append(0.0)
            continue
        wi = min(int(w), wmax)
        trans = 0.0 if (cached is not None and cached[e]) else trans_time
        t_gpu.append(max(trans, gpu_compute[wi]))
        t_cpu.append(cpu_compute[wi])
    return t_gpu, t_cpu


def greedy_assign(t_gpu: Sequence[float], t_cpu: Sequence[float]):
    """Alg. 1.  Returns (C, G, T_cpu, T_gpu)."""
    N = len(t_gpu)
    C, G = [0] * N, [0] * N
    T_cpu = T_gpu = 0.0
    sorted_indices = sorted(range(N), key=lambda i: -abs(t_gpu[i] - t_cpu[i]))      # stable: ties keep index order
    for idx in sorted_indices:
        gpu_time, cpu_time = t_gpu[idx], t_cpu[idx]
        if gpu_time == 0 and cpu_time == 0:
            continue                                                                # not activated
        if T_gpu + gpu_time <= T_cpu + cpu_time:
            G[idx] = 1
            T_gpu += gpu_time
        else:
            C[idx] = 1
            T_cpu += cpu_time
    return C, G, T_cpu, T_gpu


def optimal_assign(t_gpu: Sequence[float], t_cpu: Sequence[float]):
    """Exact minimum of max(T_gpu, T_cpu) over all assignments of the activated experts (the paper's 0-1 program
    without the memory constraint), by enumeration.  Only for small N."""
    act = [i for i in range(len(t_gpu)) if not (t_gpu[i] == 0 and t_cpu[i] == 0)]
    best = None
    for bits in range(1 << len(act)):
        Tg = sum(t_gpu[i] for j, i in enumerate(act) if bits >> j & 1)
        Tc = sum(t_cpu[i] for j, i in enumerate(act) if not bits >> j & 1)
        m = max(Tg, Tc)
        if best is None or m < best:
            best = m
    return 0.0 if best is None else best


class WorkloadAwareCache:
    """Alg. 2 for one MoE layer."""

    def __init__(self, N: int, expert_on_gpu: Sequence[int], w_size: int, u_size: int, guarded: bool = False):
        self.N, self.w_size, self.u_size, self.guarded = N, w_size, u_size, guarded
        self.s = [0] * N
        self.expert_on_gpu = sorted(expert_on_gpu)
        self.expert_on_cpu = [e for e in range(N) if e not in set(expert_on_gpu)]
        self.i = 0

    def step(self, workload: Sequence[int]):
        """One token: s = s + workload_i; at the end of a window swap and reset.  Returns [(evicted, loaded), ...]."""
        for k in range(self.N):
            self.s[k] += int(workload[k])
        swaps = []
        if (self.i + 1) % self.w_size == 0:
            cpu_trans = sorted(self.expert_on_cpu, key=lambda e: (-self.s[e], e))[: self.u_size]   # highest scores off the GPU
            gpu_evict = sorted(self.expert_on_gpu, key=lambda e: (self.s[e], e))[: self.u_size]    # lowest scores on the GPU
            for inc, out in zip(cpu_trans, gpu_evict):                      # the i-th evicted makes room for the i-th loaded
                if self.guarded and self.s[inc] <= self.s[out]:
                    break
                swaps.append((out, inc))
            for out, inc in swaps:
                self.expert_on_gpu.remove(out)
                self.expert_on_gpu.append(inc)
                self.expert_on_cpu.remove(inc)
                self.expert_on_cpu.append(out)
            self.expert_on_gpu.sort()
            self.expert_on_cpu.sort()
            self.s = [0] * self.N
        self.i += 1
        return swaps
