"""Oracle for the variable-batch dynamic program (Sec. V-C "Dynamic Programming").

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Notation follows the paper: layers L_1..L_f, Time(i,B), IN(i,B), OUT(i,B), WS(i),
TOT, and the table OPT(i,B,A) = least time to run L_1..L_i when L_i uses batch B
and A units of memory are reserved for the later layers.

READINGS
* IN and OUT grow linearly with the batch (they are activation buffers), so they
  are given per image; IN(i, B - b) in the recurrence needs batch counts that are
  not themselves candidate batch sizes.
* Memory is tracked in whole steps of ``mem_step`` bytes (the paper's table is
  indexed "in steps of 100KB"); a reservation is rounded UP to the next step.
* Candidate b for layer i-1 are the members of the batch set that divide B
  (the paper's simplification "b divides B") and are <= B.
* The latency extension: an entry whose time exceeds the threshold becomes
  infinite.
"""
from __future__ import annotations

from functools import lru_cache

INF = float("inf")


def _units(nbytes: int, step: int) -> int:
    return -(-int(nbytes) // int(step))


def plan_batches(time_ms, batch_set, in_bytes, out_bytes, ws_bytes, tot_bytes, mem_step, latency_cap_ms=None):
    """time_ms[i][j] = Time(i+1, batch_set[j]).  in_bytes / out_bytes: per image,
    per layer.  Returns (ms_per_image, [batch per layer]) or (inf, None)."""
    f = len(time_ms)
    bs = [int(b) for b in batch_set]
    col = {b: j for j, b in enumerate(bs)}
    cap = INF if latency_cap_ms is None else float(latency_cap_ms)

    def feasible(i, B, A):
        return A * mem_step + B * in_bytes[i] + ws_bytes[i] + B * out_bytes[i] <= tot_bytes

    @lru_cache(maxsize=None)
    def opt(i, B, A):
        """-> (time, chain tuple for layers 0..i)"""
        if not feasible(i, B, A):
            return INF, None
        t = float(time_ms[i][col[B]])
        if i == 0:
            return ((t, (B,)) if t <= cap else (INF, None))
        best, arg = INF, None
        for b in bs:
            if b > B or B % b:
                continue
            A2 = _units(A * mem_step + (B - b) * in_bytes[i], mem_step)
            sub, chain = opt(i - 1, b, A2)
            if sub == INF:
                continue
            c = (B // b) * sub
            if c < best:
                best, arg = c, chain + (B,)
        if arg is None:
            return INF, None
        tot = t + best
        if tot > cap:
            return INF, None
        return tot, arg

    best, plan = INF, None
    for B in bs:
        c, chain = opt(f - 1, B, 0)
        if c == INF:
            continue
        if c / B < best:
            best, plan = c / B, list(chain)
    return best, plan


def fixed_batch_baseline(time_ms, batch_set, in_bytes, out_bytes, ws_bytes, tot_bytes, latency_cap_ms=None):
    """Sec. VI baseline: one batch size for every layer, feasible at every layer,
    with the best throughput among the feasible ones."""
    f = len(time_ms)
    cap = INF if latency_cap_ms is None else float(latency_cap_ms)
    best, arg = INF, None
    for j, B in enumerate(batch_set):
        if any(B * in_bytes[i] + ws_bytes[i] + B * out_bytes[i] > tot_bytes for i in range(f)):
            continue
        t = sum(float(time_ms[i][j]) for i in range(f))
        if t > cap:
            continue
        if t / B < best:
            best, arg = t / B, int(B)
    return best, arg
