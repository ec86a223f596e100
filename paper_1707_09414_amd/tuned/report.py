"""Latency per message size and rank count from a tuner log.

    python -m paper_1707_09414_amd.tuned.report [--log SWEEP.txt] [--ranks 8,64]

Reads the candidate log ``bcast_tune`` writes (``make_table --log``; default:
the MI355X log shipped beside this file) and prints, for every rank count and
message size, the best measured time of each algorithm in microseconds, the
chain's effective bandwidth 2(P-1)M/t, and the winner -- the table behind the
paper's latency-versus-size plots (Sec. V-B) and its tuning framework.
"""
from __future__ import annotations

import argparse
import os
import sys
from collections import defaultdict

NAMES = {1: "chain", 2: "direct", 3: "binomial", 4: "fanout", 5: "scatter_allgather", 6: "knomial", 7: "knomial_pipelined"}
ORDER = [1, 7, 6, 3, 2, 5, 4]


def read(path):
    best = defaultdict(dict)  # (nranks, bytes) -> {algo: (usec, chunk, stages, trip)}
    with open(path) as f:
        for line in f:
            if not line.strip() or line.startswith("#"):
                continue
            cols = line.split()
            n, M, algo, C, stages = (int(x) for x in cols[:5])
            us = float(cols[5])
            trip = int(cols[6]) if len(cols) > 6 else 0
            rank_waves = int(cols[7]) if len(cols) > 7 else 0
            store = int(cols[8]) if len(cols) > 8 else 0
            lanes = int(cols[9]) if len(cols) > 9 else 0
            spans = int(cols[10]) if len(cols) > 10 else 0
            cur = best[(n, M)].get(algo)
            if cur is None or us < cur[0]:
                best[(n, M)][algo] = (us, C, stages, trip, rank_waves, store, lanes, spans)
    return best


def size_name(M):
    for unit, shift in (("GiB", 30), ("MiB", 20), ("KiB", 10)):
        if M >= 1 << shift:
            return "%d %s" % (M >> shift, unit)
    return "%d B" % M


def report(path, ranks=None):
    best = read(path)
    algos = [a for a in ORDER if any(a in v for v in best.values())]
    out = []
    for n in sorted({k[0] for k in best}):
        if ranks and n not in ranks:
            continue
        out.append("P = %d   (best time per algorithm in us; chain setting = chunk / stages / trip bytes / a wavefront per stage or per rank [/ stage stores written back] [/ lanes] [/ unequal stages fixed or rotating])" % n)
        out.append("%9s " % "bytes" + " ".join("%17s" % NAMES[a] for a in algos) + "  %9s  %-17s %s" % ("chain GB/s", "winner", "chain setting"))
        for M in sorted(k[1] for k in best if k[0] == n):
            row = best[(n, M)]
            win = min(row, key=lambda a: row[a][0])
            cells = " ".join("%17s" % ("%.2f" % row[a][0] if a in row else "-") for a in algos)
            c = row.get(1)
            gbs = "%9.1f" % (2.0 * (n - 1) * M / c[0] / 1e3) if c else "%9s" % "-"
            setting = "%d / %d / %d / %s%s%s%s" % (c[1], c[2], c[3], "rank" if c[4] else "stage", " / back" if c[5] == 2 else "",
                                                 " / %d lanes" % c[6] if c[6] else "", ("", " / fixed", " / rotating")[c[7]]) if c else ""
            out.append("%9s %s  %s  %-17s %s" % (size_name(M), cells, gbs, NAMES[win], setting))
        out.append("")
    return "\n".join(out)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--log", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "sweep_mi355x.txt"))
    ap.add_argument("--ranks", default="")
    args = ap.parse_args()
    ranks = {int(x) for x in args.ranks.split(",") if x}
    print(report(args.log, ranks))
    return 0


if __name__ == "__main__":
    sys.exit(main())
