"""Batch sizing of the paper's Coordinator (section 5): the package's host logic against the oracle's
brute force, and the oracle against what the equations fix."""
import numpy as np
import pytest

import oracle
from paper_2604_16400_amd import coordinator as co


def test_oracle_plane_fit_recovers_an_exact_plane_and_matches_lstsq():
    rng = np.random.default_rng(3)
    B = rng.integers(64, 4096, size=40).astype(float)
    b = rng.integers(1, 1024, size=40).astype(float)
    T = 3.5e-7 * B + 1.25e-7 * b + 4.2e-5
    c = oracle.fit_plane(B, b, T)
    assert np.allclose(c, (3.5e-7, 1.25e-7, 4.2e-5), rtol=1e-9, atol=0)
    noisy = T * (1 + 0.05 * rng.normal(size=40))
    ref, *_ = np.linalg.lstsq(np.stack([B, b, np.ones(40)], 1), noisy, rcond=None)
    assert np.allclose(oracle.fit_plane(B, b, noisy), ref, rtol=1e-8, atol=1e-16)


def test_oracle_choice_hand_example():
    # T_infer = 1 b + 2 B + 10 <= 100, T_train = 1 B + 0 b + 10, a p l = 2, B0 = 2, B in {10, 20, 30, 40, 50}
    # b*(B) = 90 - 2 B: 70, 50, 30, 10, (B = 50: -10 -> infeasible)
    # GOODPUT = B / (B + 10) * 4 / (2 + B): B=10: 0.5*4/12 = 1/6; B=20: (2/3)(4/22) = 4/33; smaller after that
    got = oracle.coordinator_choice((1.0, 0.0, 10.0), (2.0, 1.0, 10.0), 100.0, [10, 20, 30, 40, 50], 1000, 1.0, 2.0, 1.0, 2.0)
    assert got[0] == 10 and got[1] == 70 and abs(got[2] - 1.0 / 6.0) < 1e-15
    # a budget nothing meets
    assert oracle.coordinator_choice((1.0, 0.0, 10.0), (2.0, 1.0, 10.0), 5.0, [10, 20], 100, 1.0, 2.0, 1.0, 2.0) is None
    # b* is capped by b_max
    got = oracle.coordinator_choice((1.0, 0.0, 10.0), (2.0, 1.0, 10.0), 100.0, [10], 16, 1.0, 2.0, 1.0, 2.0)
    assert got[:2] == (10, 16)
    # with a large a p l the efficiency term flattens and throughput B / (B + 10) decides: the largest feasible B
    got = oracle.coordinator_choice((1.0, 0.0, 10.0), (2.0, 1.0, 10.0), 100.0, [10, 20, 30, 40, 50], 1000, 1e9, 1.0, 1.0, 2.0)
    assert got[0] == 40 and got[1] == 10


def test_package_logic_equals_oracle_on_random_models():
    rng = np.random.default_rng(20260416)
    for _ in range(300):
        tr = (rng.uniform(1e-7, 1e-6), rng.uniform(0, 5e-7), rng.uniform(1e-5, 1e-4))
        inf = (rng.uniform(0, 5e-7), rng.uniform(1e-8, 1e-6), rng.uniform(1e-5, 1e-4))
        tau = rng.uniform(5e-5, 2e-3)
        grid = list(range(64, 2049, 64))
        b_max = int(rng.integers(1, 3000))
        a, p, l, B0 = rng.uniform(0.1, 10), rng.uniform(1, 500), rng.uniform(0.01, 2), float(rng.choice([64, 128, 256]))
        ref = oracle.coordinator_choice(tr, inf, tau, grid, b_max, a, p, l, B0)
        got = co.choose_batch_sizes(co.LatencyModel(*tr), co.LatencyModel(*inf), tau, grid, b_max, a, p, l, B0)
        if ref is None:
            assert got is None
        else:
            assert got[:2] == ref[:2] and abs(got[2] - ref[2]) <= 1e-12 * abs(ref[2])


def test_package_logic_equals_oracle_on_planes_of_any_slope():
    # planes fitted to noisy timings may have coefficients of either sign (or zero): the sizing still has to be
    # the brute force's
    rng = np.random.default_rng(99)
    for _ in range(400):
        tr = (rng.uniform(-2e-7, 1e-6), rng.uniform(-2e-7, 5e-7), rng.uniform(-1e-5, 1e-4))
        inf = (rng.uniform(-2e-7, 5e-7), float(rng.choice([0.0, rng.uniform(-5e-7, 1e-6)])), rng.uniform(-1e-5, 1e-4))
        tau = rng.uniform(-1e-5, 1e-3)
        grid = list(range(64, 2049, 192))
        b_max = int(rng.integers(0, 1500))
        ref = oracle.coordinator_choice(tr, inf, tau, grid, b_max, 1.0, 100.0, 1.0, 128.0)
        got = co.choose_batch_sizes(co.LatencyModel(*tr), co.LatencyModel(*inf), tau, grid, b_max, 1.0, 100.0, 1.0, 128.0)
        if ref is None:
            assert got is None
        else:
            assert got[:2] == ref[:2] and abs(got[2] - ref[2]) <= 1e-12 * abs(ref[2])


def test_package_fit_equals_oracle():
    rng = np.random.default_rng(8)
    B = rng.integers(64, 4096, size=25).astype(float)
    b = rng.integers(1, 1024, size=25).astype(float)
    T = (3e-7 * B + 1e-7 * b + 5e-5) * (1 + 0.02 * rng.normal(size=25))
    m, r2 = co.fit_latency_model(B, b, T)
    assert np.allclose((m.coef_B, m.coef_b, m.const), oracle.fit_plane(B, b, T), rtol=1e-8, atol=1e-16)
    assert 0.9 < r2 <= 1.0


@pytest.mark.gpu
def test_measured_planes_feed_the_same_choice_as_the_oracle():
    """The sweep that feeds the model, on the GPU: a 3 x 3 grid of (training tokens, decode tokens) on a small layer,
    the planes fitted to what was measured, and the batch sizing on them equal to the oracle's brute force."""
    Bg, bg = (512, 1024, 2048), (128, 512, 1024)
    rows = co.measure(d_in=2048, d_out=2048, n_adapters=8, rank=16, B_grid=Bg, b_grid=bg, iters=5)
    assert [(r["B"], r["b"]) for r in rows] == [(B, b) for B in Bg for b in bg]
    Bv, bv = [r["B"] for r in rows], [r["b"] for r in rows]
    for r in rows:
        assert all(np.isfinite(r[k]) and 0 < r[k] < 0.1 for k in ("fused_s", "streams_train_s", "streams_infer_s"))
    # (no claim about the timings themselves beyond being sane: what is tested is the arithmetic on whatever was measured)
    fits = {}
    for key in ("fused_s", "streams_train_s", "streams_infer_s"):
        T = [r[key] for r in rows]
        m, r2 = co.fit_latency_model(Bv, bv, T)
        ref = oracle.fit_plane(Bv, bv, T)
        assert np.allclose((m.coef_B, m.coef_b, m.const), ref, rtol=1e-6, atol=1e-12)
        fits[key] = m
    tau = 2.0 * min(r["fused_s"] for r in rows)
    grid = list(range(256, 2049, 128))
    for train, infer in ((fits["fused_s"], fits["fused_s"]), (fits["streams_train_s"], fits["streams_infer_s"])):
        got = co.choose_batch_sizes(train, infer, tau, grid, 1024, 1.0, 2048.0, 1.0, 1024.0)
        ref = oracle.coordinator_choice((train.coef_B, train.coef_b, train.const), (infer.coef_B, infer.coef_b, infer.const),
                                        tau, grid, 1024, 1.0, 2048.0, 1.0, 1024.0)
        if ref is None:
            assert got is None
        else:
            assert got[:2] == ref[:2] and abs(got[2] - ref[2]) <= 1e-9 * abs(ref[2])
