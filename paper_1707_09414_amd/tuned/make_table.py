"""Measure the tuning table on the GPU in this machine and write it as text.

    python -m paper_1707_09414_amd.tuned.make_table [--out PATH] [--ranks 2,4,8,...]
                                                    [--min-bytes N] [--max-bytes N] [--with-fanout] [--with-knomial] [--with-knomial-pipelined]
                                                    [--with-scatter-allgather] [--folded] [--no-rank-waves] [--append]
                                                    [--reduce] [--reduce-only]

For every rank count it runs ``bcast_tune`` (chain over chunk sizes, stage counts and
trip sizes, with a wavefront per stage and with a wavefront per rank, direct, binomial;
the one-die fan-out and the single-stage chain only on request) over power-of-two message sizes
and writes the winners.  The file it produces is what ``load_default_table``
installs.
"""
from __future__ import annotations

import argparse
import os
import sys
import time


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "mi355x.txt"))
    ap.add_argument("--ranks", default="2,4,8,16,32,64")
    ap.add_argument("--min-bytes", type=int, default=4)
    ap.add_argument("--max-bytes", type=int, default=1 << 30)
    ap.add_argument("--with-fanout", action="store_true")
    ap.add_argument("--with-knomial", action="store_true", help="also try the k-nomial tree at radix 4 and 8")
    ap.add_argument("--with-knomial-pipelined", action="store_true",
                    help="also try the one-launch pipelined k-nomial tree at radix 2, 4, 8, 16 and the rank count")
    ap.add_argument("--with-scatter-allgather", action="store_true")
    ap.add_argument("--log", default=None, help="also append every timed candidate to this file")
    ap.add_argument("--folded", action="store_true", help="also try the chain with a single stage (no flag hand-off)")
    ap.add_argument("--no-rank-waves", action="store_true", help="leave out the chain with a wavefront per rank")
    ap.add_argument("--reduce", action="store_true", help="also measure the chain reduction's table (bcast_tune_reduce)")
    ap.add_argument("--reduce-only", action="store_true", help="measure only the chain reduction's table")
    ap.add_argument("--append", action="store_true", help="keep the entries --out already holds (other rank counts)")
    args = ap.parse_args()

    import torch  # device context and stream only

    from .. import binding as B

    torch.cuda.set_device(0)
    mask = (1 << B.BCAST_ALGO_CHAIN) | (1 << B.BCAST_ALGO_DIRECT) | (1 << B.BCAST_ALGO_BINOMIAL)
    if args.with_fanout:
        mask |= 1 << B.BCAST_ALGO_FANOUT
    if args.with_knomial:
        mask |= 1 << B.BCAST_ALGO_KNOMIAL
    if args.with_knomial_pipelined:
        mask |= 1 << B.BCAST_ALGO_KNOMIAL_PIPELINED
    if args.with_scatter_allgather:
        mask |= 1 << B.BCAST_ALGO_SCATTER_ALLGATHER
    if args.folded:
        mask |= B.BCAST_TUNE_FOLDED
    if args.no_rank_waves:
        mask |= B.BCAST_TUNE_NO_RANK_WAVES
    B.bcast_tune_clear()
    if args.append and os.path.exists(args.out):
        B.bcast_tune_load(args.out)
    B.bcast_tune_set_log(args.log)
    stream = torch.cuda.current_stream()
    for P in [int(x) for x in args.ranks.split(",")]:
        t0 = time.time()
        if not args.reduce_only:
            B.bcast_tune(P, args.min_bytes, args.max_bytes, mask, stream, None)
            print("tuned P=%d in %.1f s (%d entries so far)" % (P, time.time() - t0, B.bcast_tune_count()), flush=True)
        if args.reduce or args.reduce_only:
            t0 = time.time()
            B.bcast_tune_reduce(P, max(4, args.min_bytes), args.max_bytes, stream, None)
            print("tuned the reduction for P=%d in %.1f s" % (P, time.time() - t0), flush=True)
    B.bcast_tune_set_log(None)
    B.bcast_tune_save(args.out)
    print("wrote", args.out)
    return 0


if __name__ == "__main__":
    sys.exit(main())
