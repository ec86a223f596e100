"""The paper's cost models (Sec. III-A Eq. 1-4, Sec. IV-B Eq. 5) and their fit
to measured broadcast times.

    python -m paper_1707_09414_amd.model --log SWEEP.txt [--ranks 8]

`SWEEP.txt` is what ``bcast_tune`` writes while a log path is set
(``make_table --log``): one line per timed candidate,
``nranks bytes algo chunk_bytes stages usec [trip_bytes]``.  For every rank count the start-up
time t_s and the bandwidth B of Table I are estimated per algorithm by linear
least squares (each model is linear in t_s and 1/B), the model's prediction is
compared with every measurement, and the chunk size that minimises Eq. 5,
C* = sqrt(M t_s B / (n - 2)), is set beside the measured best chunk.

This module only needs numpy; it runs on a machine without a GPU.
"""
from __future__ import annotations

import argparse
import math
import sys
from collections import defaultdict
from typing import Dict, Iterable, List, Tuple

import numpy as np

ALGO_CHAIN, ALGO_DIRECT, ALGO_BINOMIAL, ALGO_FANOUT = 1, 2, 3, 4
ALGO_KNOMIAL, ALGO_KNOMIAL_PIPELINED = 6, 7


def ceil_log(n: int, k: int) -> int:
    """Smallest r with k**r >= n."""
    r, reach = 0, 1
    while reach < n:
        reach *= k
        r += 1
    return r


# ---- the models, as printed -------------------------------------------------

def t_direct(n, M, ts, B):
    """Eq. 1: n (t_s + M/B)."""
    return n * (ts + M / B)


def t_chain(n, M, ts, B):
    """Eq. 2: (n - 1)(t_s + M/B)."""
    return (n - 1) * (ts + M / B)


def t_knomial(n, k, M, ts, B):
    """Eq. 3: ceil(log_k n)(t_s + M/B)."""
    return ceil_log(n, k) * (ts + M / B)


def t_scatter_allgather(n, M, ts, B):
    """Eq. 4: (ceil(log2 n) + n - 1) t_s + 2 (n - 1)/n M/B."""
    return (ceil_log(n, 2) + n - 1) * ts + 2.0 * ((n - 1) * M / n) / B


def t_chain_pipeline(n, M, C, ts, B):
    """Eq. 5: (M/C + n - 2)(t_s + C/B)."""
    return (M / C + (n - 2)) * (ts + C / B)


def t_knomial_pipeline(n, k, M, C, ts, B):
    """This build's extension of Eq. 5's chunking to the tree of Eq. 3, level by
    level: a level is done when its senders have pushed all M/C chunks to their
    children, one chunk per step of (t_s + C/B), and there are ceil(log_k n)
    levels: (M/C ceil(log_k n))(t_s + C/B).  Not a formula of the paper."""
    return (M / C * ceil_log(n, k)) * (ts + C / B)


def best_chunk(n, M, ts, B):
    """Minimiser of Eq. 5 over C (own derivation): sqrt(M t_s B / (n - 2))."""
    if n <= 2:
        return float(M)
    return math.sqrt(M * ts * B / (n - 2))


# ---- fitting ------------------------------------------------------------------

def _lstsq(rows: List[Tuple[float, float]], y: List[float]) -> Tuple[float, float]:
    """Solve y ~ a * x0 + b * x1 for (a, b) = (t_s, 1/B), weighting every point by
    1/y so that small and large messages count alike (relative error)."""
    A = np.array(rows, dtype=np.float64)
    t = np.array(y, dtype=np.float64)
    w = 1.0 / t
    sol, *_ = np.linalg.lstsq(A * w[:, None], t * w, rcond=None)
    return float(sol[0]), float(sol[1])


def fit_steps_model(points: Iterable[Tuple[float, float, float]]) -> Tuple[float, float]:
    """Fit T = steps * (t_s + bytes_per_step / B) to (steps, bytes_per_step, T)
    triples; every model above has this shape.  Returns (t_s, B)."""
    rows, y = [], []
    for steps, per_step, T in points:
        rows.append((steps, steps * per_step))
        y.append(T)
    ts, inv_b = _lstsq(rows, y)
    return ts, (1.0 / inv_b if inv_b > 0 else float("inf"))


def steps_direct(n, M):
    """(steps, bytes per step) of the direct algorithm as the text describes it:
    one send per non-root rank (Eq. 1 prints n)."""
    return n - 1, M


def steps_binomial(n, M):
    return ceil_log(n, 2), M


def steps_chain(n, M, C):
    C = min(C, M)
    return math.ceil(M / C) + n - 2, C


def read_log(path: str) -> Dict[int, List[Tuple[int, int, int, int, float]]]:
    """{nranks: [(bytes, algo, chunk, stages, seconds)]}"""
    out: Dict[int, list] = defaultdict(list)
    with open(path) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            cols = line.split()
            n, M, algo, C, stages, us = cols[:6]
            # column 8 (newer logs): 1 = the chain ran with a wavefront per rank, whose hand-offs inside a
            # workgroup are per trip, not per chunk: Eq. 5 with chunk C models the other kernel, so those rows are left out
            if len(cols) > 7 and int(cols[7]) != 0:
                continue
            out[int(n)].append((int(M), int(algo), int(C), int(stages), float(us) * 1e-6))
    return out


def fit_rank_count(n: int, rows, min_bytes: int = 0):
    """Fit every algorithm's model for one rank count.  Chain rows are those with
    one stage per receiving rank (stages == n - 1), the structure Eq. 5 models.
    Returns {name: dict(ts, B, n_points, rel_err_mean, rel_err_max)} and a list of
    (M, measured best C, C* from the fit)."""
    groups = {"direct": [], "binomial": [], "chain": []}
    for M, algo, C, stages, T in rows:
        if M < min_bytes:
            continue
        if algo == ALGO_DIRECT:
            groups["direct"].append((*steps_direct(n, M), T))
        elif algo == ALGO_BINOMIAL:
            groups["binomial"].append((*steps_binomial(n, M), T))
        elif algo == ALGO_CHAIN and stages == n - 1:
            groups["chain"].append((*steps_chain(n, M, C), T))
    fits = {}
    for name, pts in groups.items():
        if len(pts) < 2:
            continue
        ts, B = fit_steps_model(pts)
        errs = [abs(s * (ts + b / B) - T) / T for s, b, T in pts]
        fits[name] = dict(ts=ts, B=B, n_points=len(pts), rel_err_mean=float(np.mean(errs)), rel_err_max=float(np.max(errs)))
    chunks = []
    if "chain" in fits:
        by_M = defaultdict(list)
        for M, algo, C, stages, T in rows:
            if algo == ALGO_CHAIN and stages == n - 1 and M >= min_bytes:
                by_M[M].append((T, min(C, M)))
        for M in sorted(by_M):
            if len(by_M[M]) > 1:
                chunks.append((M, min(by_M[M])[1], best_chunk(n, M, fits["chain"]["ts"], fits["chain"]["B"])))
    return fits, chunks


def report(log_path: str, ranks=None, min_bytes: int = 0) -> str:
    data = read_log(log_path)
    lines = []
    for n in sorted(data):
        if ranks and n not in ranks:
            continue
        fits, chunks = fit_rank_count(n, data[n], min_bytes)
        lines.append("n = %d ranks" % n)
        for name in ("direct", "binomial", "chain"):
            if name in fits:
                f = fits[name]
                lines.append("  %-8s t_s = %8.3f us   B = %8.1f GB/s   points %3d   |model - measured| / measured: mean %5.1f %%, max %5.1f %%"
                             % (name, f["ts"] * 1e6, f["B"] / 1e9, f["n_points"], 100 * f["rel_err_mean"], 100 * f["rel_err_max"]))
        for M, c_meas, c_star in chunks:
            lines.append("  chain M = %11d B: measured best C = %9d B, Eq. 5 optimum C* = %11.0f B" % (M, c_meas, c_star))
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--log", required=True)
    ap.add_argument("--ranks", default="")
    ap.add_argument("--min-bytes", type=int, default=0, help="ignore smaller messages in the fit")
    args = ap.parse_args()
    ranks = {int(x) for x in args.ranks.split(",") if x}
    print(report(args.log, ranks, args.min_bytes))
    return 0


if __name__ == "__main__":
    sys.exit(main())
