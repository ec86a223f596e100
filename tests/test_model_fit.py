"""The cost-model module against the oracle's evaluation of the same printed
formulas (Sec. III-A Eq. 1-4, Sec. IV-B Eq. 5), and the fit against data
synthesised from those formulas: the planted t_s and B must come back."""
import math

import numpy as np
import pytest

import oracle
from paper_1707_09414_amd import model


@pytest.mark.parametrize("n", [2, 3, 8, 16, 33, 64])
def test_models_match_the_oracle(n):
    rng = np.random.default_rng(n)
    for _ in range(20):
        M = float(rng.integers(1, 1 << 30))
        C = float(rng.integers(1, 1 << 22))
        ts = float(rng.uniform(1e-7, 1e-4))
        Bw = float(rng.uniform(1e8, 1e13))
        assert model.t_direct(n, M, ts, Bw) == pytest.approx(oracle.model_direct(n, M, ts, Bw), rel=1e-13)
        assert model.t_chain(n, M, ts, Bw) == pytest.approx(oracle.model_chain(n, M, ts, Bw), rel=1e-13)
        for k in (2, 3, 4, 8):
            assert model.t_knomial(n, k, M, ts, Bw) == pytest.approx(oracle.model_knomial(n, k, M, ts, Bw), rel=1e-13)
            assert model.t_knomial_pipeline(n, k, M, C, ts, Bw) == pytest.approx(oracle.model_knomial_pipeline(n, k, M, C, ts, Bw), rel=1e-13)
        assert model.t_scatter_allgather(n, M, ts, Bw) == pytest.approx(oracle.model_scatter_allgather(n, M, ts, Bw), rel=1e-13)
        assert model.t_chain_pipeline(n, M, C, ts, Bw) == pytest.approx(oracle.model_chain_pipeline(n, M, C, ts, Bw), rel=1e-13)


def test_best_chunk_minimises_eq5():
    n, M, ts, Bw = 16, 64.0 * (1 << 20), 3e-6, 5e11
    c_star = model.best_chunk(n, M, ts, Bw)
    t_star = oracle.model_chain_pipeline(n, M, c_star, ts, Bw)
    for f in (0.5, 0.9, 1.1, 2.0):
        assert oracle.model_chain_pipeline(n, M, c_star * f, ts, Bw) > t_star
    assert model.best_chunk(2, M, ts, Bw) == M


def test_fit_recovers_planted_parameters(tmp_path):
    n, ts, Bw = 8, 2.5e-6, 8.0e11
    lines = ["# nranks bytes algo chunk_bytes stages usec"]
    for lg in range(12, 27):
        M = 1 << lg
        lines.append("%d %d 2 0 0 %.6f" % (n, M, 1e6 * (n - 1) * (ts + M / Bw)))
        lines.append("%d %d 3 0 0 %.6f" % (n, M, 1e6 * oracle.model_knomial(n, 2, M, ts, Bw)))
        for lc in range(13, 23):
            C = 1 << lc
            if C < M:
                nchunks = math.ceil(M / C)
                lines.append("%d %d 1 %d %d %.6f" % (n, M, C, n - 1, 1e6 * (nchunks + n - 2) * (ts + C / Bw)))
                lines.append("%d %d 1 %d 2 %.6f" % (n, M, C, 123.0))  # other stage counts are not Eq. 5's structure
    path = tmp_path / "sweep.txt"
    path.write_text("\n".join(lines) + "\n")
    fits, chunks = model.fit_rank_count(n, model.read_log(str(path))[n])
    for name in ("direct", "binomial", "chain"):
        assert fits[name]["ts"] == pytest.approx(ts, rel=1e-6), name
        assert fits[name]["B"] == pytest.approx(Bw, rel=1e-6), name
        assert fits[name]["rel_err_max"] < 1e-6
    # with exact Eq. 5 data the measured best chunk is the power of two next to C*
    for M, c_meas, c_star in chunks:
        if 8192 * 2 <= c_star <= (1 << 21) and c_star * 2 < M:
            assert 0.5 <= c_meas / c_star <= 2.0, (M, c_meas, c_star)
    text = model.report(str(path))
    assert "n = 8 ranks" in text and "chain" in text


def test_fit_of_the_committed_mi355x_sweep():
    """The measurement log shipped with the package (written by bcast_tune on an
    MI355X) must parse and give physically sensible parameters: a start-up time
    of a few microseconds per launch and terabytes per second."""
    import os

    path = os.path.join(os.path.dirname(model.__file__), "tuned", "sweep_mi355x.txt")
    data = model.read_log(path)
    assert sorted(data) == [2, 4, 8, 16, 32, 64]
    for n in data:
        fits, chunks = model.fit_rank_count(n, data[n], min_bytes=65536)
        assert 1e-6 < fits["direct"]["ts"] < 6e-6 and 1e12 < fits["direct"]["B"] < 8e12
        assert 1e-6 < fits["binomial"]["ts"] < 6e-6
        assert 0.3e-6 < fits["chain"]["ts"] < 6e-6
        if n >= 8:
            # one die: binomial's rounds do not run on separate links, so its
            # fitted per-round bandwidth falls as rounds get more crowded
            assert fits["binomial"]["B"] < fits["direct"]["B"]


def test_latency_report_of_the_committed_sweep():
    """The per-size latency table is derived from the shipped log and agrees
    with the committed text copy of it."""
    import os

    from paper_1707_09414_amd.tuned import report

    here = os.path.dirname(report.__file__)
    text = report.report(os.path.join(here, "sweep_mi355x.txt"))
    assert text.strip() == open(os.path.join(here, "latency_mi355x.txt")).read().strip()
    best = report.read(os.path.join(here, "sweep_mi355x.txt"))
    assert len(best) == 6 * 29
    # the landscape the tuning table encodes: a tree for small messages, the chain for large ones
    assert min(best[(64, 4096)], key=lambda a: best[(64, 4096)][a][0]) == 7
    assert min(best[(64, 1 << 30)], key=lambda a: best[(64, 1 << 30)][a][0]) == 1
    assert best[(64, 4096)][1][0] < best[(64, 4096)][2][0]  # the chain beats direct at P = 64
