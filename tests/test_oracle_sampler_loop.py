"""Pins for the oracle's reuse-then-predict loop (Appendix A, Algorithm 1), its batched
single-device form (Section 3.3) and the direct-reuse process (Section 3.1)."""
import math
import os

import numpy as np
import pytest

from oracle import parastep_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def scalar_predictor(x, tau):
    return np.sin(x) + tau / 1000.0


def plain_loop(predict, x, tau, a, b):
    for i in range(len(tau)):
        x = a[i] * x + b[i] * predict(x, int(tau[i]))
    return x


def test_hand_trace_S7_m1_p3():
    """Which rank evaluates at which step, written out from Algorithm 1: step 0 is
    warm-up; afterwards the evaluating rank cycles 0,1,2 and rank 0 applies its eps."""
    tau, a, b = O.ddim_coefficients(steps=7)
    trace = []
    O.run_sampler(scalar_predictor, np.array([0.3]), tau, a, b, warmup=1, cycle_len=[3, 3], trace=trace)
    assert trace == [(0, 0, 0), (1, 0, 0), (2, 1, 1), (3, 2, 2), (4, 0, 0), (5, 1, 1), (6, 2, 2)]


def test_straight_line_script_S7_m1_p3():
    """The same run as a loop-free script with one variable per tensor.

    Warm-up sets every rank's cache to e0.  In the first cycle ranks 1 and 2 advance
    with e0; in the second cycle rank 1 advances with the eps it predicted in cycle one
    (E2) and rank 2 with its own (E3): a rank's cache changes only when it predicts.
    """
    f = scalar_predictor
    tau, a, b = O.ddim_coefficients(steps=7)
    st = lambda i, x, e: a[i] * x + b[i] * e
    xT = np.array([0.3, -1.1, 2.0])
    e0 = f(xT, tau[0]);  X1 = st(0, xT, e0)
    E1 = f(X1, tau[1]);  X2 = st(1, X1, E1);  Y2 = st(1, X1, e0)
    E2 = f(Y2, tau[2]);  X3 = st(2, X2, E2);  Z3 = st(2, Y2, e0)
    E3 = f(Z3, tau[3]);  X4 = st(3, X3, E3)
    E4 = f(X4, tau[4]);  X5 = st(4, X4, E4);  Y5 = st(4, X4, E2);  Z5 = st(4, X4, E3)
    E5 = f(Y5, tau[5]);  X6 = st(5, X5, E5);  Z6 = st(5, Z5, E3)
    E6 = f(Z6, tau[6]);  X7 = st(6, X6, E6)
    out = O.run_sampler(f, xT, tau, a, b, warmup=1, cycle_len=[3, 3])
    np.testing.assert_allclose(out["x0"], X7, rtol=0, atol=1e-12)
    for got, ref in zip(out["xs"], [X1, X2, X3, X4, X5, X6, X7]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    for got, ref in zip(out["eps"], [e0, E1, E2, E3, E4, E5, E6]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    # and it is NOT the plain process (the predictor really varies)
    assert np.abs(out["x0"] - plain_loop(f, xT, tau, a, b)).max() > 1e-4


def test_straight_line_script_truncated_cycle_S6_m2_p3():
    """(S - m) not a multiple of p: the run stops mid-cycle and returns rank 0's sample."""
    f = scalar_predictor
    tau, a, b = O.ddim_coefficients(steps=6)
    st = lambda i, x, e: a[i] * x + b[i] * e
    xT = np.array([0.7])
    e0 = f(xT, tau[0]);  X1 = st(0, xT, e0)
    e1 = f(X1, tau[1]);  X2 = st(1, X1, e1)             # warm-up ends; caches = e1
    E2 = f(X2, tau[2]);  X3 = st(2, X2, E2);  Y3 = st(2, X2, e1)
    E3 = f(Y3, tau[3]);  X4 = st(3, X3, E3);  Z4 = st(3, Y3, e1)
    E4 = f(Z4, tau[4]);  X5 = st(4, X4, E4)             # broadcast
    E5 = f(X5, tau[5]);  X6 = st(5, X5, E5)             # round 0 of a cycle that never ends
    out = O.run_sampler(f, xT, tau, a, b, warmup=2, cycle_len=[3, 3])
    np.testing.assert_allclose(out["x0"], X6, rtol=0, atol=1e-12)


@pytest.mark.parametrize("S,m", [(8, 2), (7, 1), (5, 5), (5, 9)])
def test_window_one_or_all_warmup_is_the_plain_loop(S, m):
    tau, a, b = O.ddim_coefficients(steps=S)
    xT = np.linspace(-2, 2, 9)
    ref = plain_loop(scalar_predictor, xT.copy(), tau, a, b)
    out1 = O.run_sampler(scalar_predictor, xT, tau, a, b, warmup=min(m, S), cycle_len=[1] * S)
    np.testing.assert_array_equal(out1["x0"], ref)
    out2 = O.run_sampler(scalar_predictor, xT, tau, a, b, warmup=S, cycle_len=[4])
    np.testing.assert_array_equal(out2["x0"], ref)
    assert out1["calls"] == S and out2["calls"] == S


@pytest.mark.parametrize("p,m", [(2, 1), (3, 2), (4, 1), (4, 3)])
def test_constant_predictor_gives_the_closed_form_for_every_window(p, m):
    S = 12
    tau, a, b = O.ddim_coefficients(steps=S)
    ab = O.ddim_alphas_cumprod()
    rng = np.random.default_rng(0)
    xT, e = rng.standard_normal(6), rng.standard_normal(6)
    out = O.run_sampler(lambda x, t: e, xT, tau, a, b, warmup=m, cycle_len=[p] * S)
    ref = (xT - math.sqrt(1 - ab[tau[0]]) * e) / math.sqrt(ab[tau[0]])
    np.testing.assert_allclose(out["x0"], ref, atol=1e-10)
    assert out["re"][1:] == [0.0] * (S - 1)


@pytest.mark.parametrize("p,m", [(2, 1), (3, 1), (4, 2)])
def test_point_mass_predictor_makes_reuse_exact(p, m):
    """eps = x / sqrt(1-abar_tau) is constant along its own trajectory, so every reused
    eps is the true one and the result equals the plain process."""
    S = 10
    tau, a, b = O.ddim_coefficients(steps=S)
    ab = O.ddim_alphas_cumprod()
    f = lambda x, t: x / math.sqrt(1 - ab[t])
    xT = np.random.default_rng(1).standard_normal(5)
    out = O.run_sampler(f, xT, tau, a, b, warmup=m, cycle_len=[p] * S)
    ref = plain_loop(f, xT.copy(), tau, a, b)
    np.testing.assert_allclose(out["x0"], ref, atol=1e-12)
    for i in range(S - 1):
        np.testing.assert_allclose(out["xs"][i], xT * math.sqrt(1 - ab[tau[i + 1]]) / math.sqrt(1 - ab[tau[0]]),
                                   atol=1e-12)


@pytest.mark.parametrize("S,m,cyc", [(7, 1, [3, 3]), (8, 2, [2, 2, 2]), (9, 2, [4, 4]), (10, 1, [1, 2, 4, 2]),
                                     (6, 2, [3, 3])])
def test_batched_form_equals_the_rank_simulation(S, m, cyc):
    tau, a, b = O.ddim_coefficients(steps=S)
    xT = np.random.default_rng(2).standard_normal(4)
    ref = O.run_sampler(scalar_predictor, xT, tau, a, b, warmup=m, cycle_len=cyc)
    fb = lambda xb, ts: np.stack([scalar_predictor(xb[i], int(ts[i])) for i in range(len(ts))])
    out = O.run_sampler_batched(fb, xT, tau, a, b, warmup=m, cycle_len=cyc)
    np.testing.assert_allclose(out["x0"], ref["x0"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(out["rx"], ref["rx"], rtol=1e-12)
    np.testing.assert_allclose(out["re"][1:], ref["re"][1:], rtol=1e-10)
    # the batched form makes one call per warm-up step and one per cycle
    assert ref["calls"] == S
    assert out["calls"] == m + len(O.expand_cycles(S, m, cyc))


def test_reuse_ages_own_cache_and_latest_eps():
    """How old the reused eps is, from the structure of Algorithm 1 alone.  A cycle of
    length p starts at step c; rank r (1 <= r < p) makes reuse updates at steps c..c+r-1.
    With its own cache the eps was predicted at step c-p+r (the previous cycle's round
    r), or at the last warm-up step in the first cycle.  In the latest-eps variant it is
    the eps of step c-1, whatever the rank."""
    S, m, p = 11, 2, 3
    tau, a, b = O.ddim_coefficients(steps=S)
    own, latest = [], []
    O.run_sampler(scalar_predictor, np.array([0.1]), tau, a, b, m, [p] * 3, reuse_trace=own)
    O.run_sampler(scalar_predictor, np.array([0.1]), tau, a, b, m, [p] * 3, mode="latest_eps", reuse_trace=latest)
    exp_own, exp_latest = [], []
    for c in (2, 5, 8):
        for j in range(p):                    # round j: ranks j+1..p-1 reuse at step c+j
            for r in range(j + 1, p):
                exp_own.append((c + j, r, m - 1 if c == m else c - p + r))
                exp_latest.append((c + j, r, c - 1))
    assert sorted(own) == sorted(exp_own)
    assert sorted(latest) == sorted(exp_latest)


def test_latest_eps_straight_line_script_S7_m1_p3():
    """Loop-free script of the latest-eps variant: the first cycle is that of Algorithm 1
    (every cache holds e0); in the second cycle ranks 1 and 2 advance with E3, the eps of
    the step before the cycle, instead of E2 and E3."""
    f = scalar_predictor
    tau, a, b = O.ddim_coefficients(steps=7)
    st = lambda i, x, e: a[i] * x + b[i] * e
    xT = np.array([0.3, -1.1, 2.0])
    e0 = f(xT, tau[0]);  X1 = st(0, xT, e0)
    E1 = f(X1, tau[1]);  X2 = st(1, X1, E1);  Y2 = st(1, X1, e0)
    E2 = f(Y2, tau[2]);  X3 = st(2, X2, E2);  Z3 = st(2, Y2, e0)
    E3 = f(Z3, tau[3]);  X4 = st(3, X3, E3)
    E4 = f(X4, tau[4]);  X5 = st(4, X4, E4);  Y5 = st(4, X4, E3);  Z5 = st(4, X4, E3)
    E5 = f(Y5, tau[5]);  X6 = st(5, X5, E5);  Z6 = st(5, Z5, E3)
    E6 = f(Z6, tau[6]);  X7 = st(6, X6, E6)
    out = O.run_sampler(f, xT, tau, a, b, warmup=1, cycle_len=[3, 3], mode="latest_eps")
    for got, ref in zip(out["xs"], [X1, X2, X3, X4, X5, X6, X7]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    for got, ref in zip(out["eps"], [e0, E1, E2, E3, E4, E5, E6]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    own = O.run_sampler(f, xT, tau, a, b, warmup=1, cycle_len=[3, 3])
    assert np.abs(out["x0"] - own["x0"]).max() > 1e-6          # the two variants differ at p = 3


@pytest.mark.parametrize("S,m", [(9, 1), (10, 2)])
def test_latest_eps_equals_algorithm_1_for_cycles_of_two(S, m):
    """With p = 2 the only reuse update is rank 1's at round 0, and its own cache is the
    eps of the step before the cycle: both variants are the same process."""
    tau, a, b = O.ddim_coefficients(steps=S)
    xT = np.random.default_rng(5).standard_normal(6)
    r0 = O.run_sampler(scalar_predictor, xT, tau, a, b, m, [2] * S)
    r1 = O.run_sampler(scalar_predictor, xT, tau, a, b, m, [2] * S, mode="latest_eps")
    np.testing.assert_array_equal(r0["x0"], r1["x0"])
    np.testing.assert_array_equal(np.stack(r0["xs"]), np.stack(r1["xs"]))


@pytest.mark.parametrize("S,m,cyc", [(7, 1, [3, 3]), (9, 2, [4, 4]), (10, 1, [1, 2, 4, 2]), (12, 2, [2, 4, 8]),
                                     (11, 3, [8])])
def test_latest_eps_batched_form_equals_the_rank_simulation(S, m, cyc):
    tau, a, b = O.ddim_coefficients(steps=S)
    xT = np.random.default_rng(3).standard_normal(4)
    ref = O.run_sampler(scalar_predictor, xT, tau, a, b, warmup=m, cycle_len=cyc, mode="latest_eps")
    fb = lambda xb, ts: np.stack([scalar_predictor(xb[i], int(ts[i])) for i in range(len(ts))])
    out = O.run_sampler_batched(fb, xT, tau, a, b, warmup=m, cycle_len=cyc, mode="latest_eps")
    np.testing.assert_allclose(out["x0"], ref["x0"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(out["rx"], ref["rx"], rtol=1e-12)
    assert out["calls"] == m + len(O.expand_cycles(S, m, cyc))


def test_direct_reuse_is_the_plain_loop_on_the_coarser_grid():
    """Stride-2 direct reuse after one warm-up step equals DDIM whose steps 1.. are
    merged in pairs (jump consistency of the update)."""
    f = scalar_predictor
    tau, a, b = O.ddim_coefficients(steps=7)
    xT = np.array([0.2, 1.4])
    out = O.run_sampler(f, xT, tau, a, b, warmup=1, cycle_len=[2, 2, 2], mode="direct_reuse")
    x = a[0] * xT + b[0] * f(xT, tau[0])
    for i in (1, 3, 5):
        e = f(x, tau[i])
        x = a[i + 1] * (a[i] * x + b[i] * e) + b[i + 1] * e
    np.testing.assert_allclose(out["x0"], x, atol=1e-13)
    assert out["calls"] == 4


def test_per_step_records():
    tau, a, b = O.ddim_coefficients(steps=8)
    xT = np.random.default_rng(3).standard_normal(7)
    out = O.run_sampler(scalar_predictor, xT, tau, a, b, warmup=2, cycle_len=[2] * 3)
    prev = xT
    for i in range(8):
        assert out["rx"][i] == pytest.approx(np.abs(out["xs"][i] - prev).sum() / np.abs(out["xs"][i]).sum(), rel=1e-13)
        prev = out["xs"][i]
    assert math.isnan(out["re"][0])
    assert out["re"][3] == pytest.approx(np.abs(out["eps"][3] - out["eps"][2]).sum() / np.abs(out["eps"][3]).sum(),
                                         rel=1e-13)


def test_no_warmup_with_window_is_rejected():
    tau, a, b = O.ddim_coefficients(steps=4)
    with pytest.raises(ValueError):
        O.run_sampler(scalar_predictor, np.zeros(2), tau, a, b, warmup=0, cycle_len=[2, 2])
    with pytest.raises(ValueError):
        O.run_sampler(scalar_predictor, np.zeros(2), tau, a, b, warmup=1, cycle_len=[2])   # does not cover


def test_critical_path_against_the_papers_bound_and_measurements():
    """Each device evaluates the predictor once per cycle, so its critical path is
    m + ceil((S-m)/p) evaluations; S over that is the paper's bound when p divides S-m,
    and every speedup the paper measured lies below the bound."""
    assert O.critical_path_calls(50, 13, 2) == 32
    assert O.critical_path_calls(50, 50, 4) == 50 and O.critical_path_calls(8, 2, 2) == 5
    assert 50 / O.critical_path_calls(50, 10, 4) == pytest.approx(O.amdahl_bound(10 / 50, 4), rel=1e-14)
    assert O.amdahl_bound(0.0, 8) == 8.0 and O.amdahl_bound(1.0, 8) == 1.0
    rows = 0
    with open(os.path.join(HERE, "golden", "paper_speedups.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            model, S, m, p, t_orig, t_para = line.split()
            S, m, p = int(S), int(m), int(p)
            measured = float(t_orig) / float(t_para)
            assert 1.0 < measured < O.amdahl_bound(m / S, p), model
            assert measured < S / O.critical_path_calls(S, m, p) + 1e-12, model
            rows += 1
    assert rows == 9


@pytest.mark.parametrize("mode", ["reuse_then_predict", "latest_eps", "direct_reuse"])
@pytest.mark.parametrize("S,m,cyc", [(7, 1, [3, 3]), (10, 1, [1, 2, 4, 2]), (8, 2, [2, 2, 2]), (6, 2, [3, 3])])
def test_a_run_in_two_pieces_is_the_whole_run(mode, S, m, cyc):
    """Stopping after any step and continuing from the returned state (step, cycle, round, every rank's
    sample and eps_cache, last eps) reproduces the uninterrupted run bit for bit."""
    tau, a, b = O.ddim_coefficients(steps=S)
    xT = np.array([0.3, -1.1, 2.0, 0.7])
    whole = O.run_sampler(scalar_predictor, xT, tau, a, b, m, cyc, mode=mode)
    for k in range(1, S):
        one = O.run_sampler(scalar_predictor, xT, tau, a, b, m, cyc, mode=mode, stop=k)
        assert one["state"]["step"] == k and len(one["xs"]) == k
        two = O.run_sampler(scalar_predictor, xT, tau, a, b, m, cyc, mode=mode, state=one["state"])
        assert np.array_equal(two["x0"], whole["x0"])
        assert one["calls"] <= two["calls"] == whole["calls"]          # (direct reuse: a piece may hold no prediction)
        for got, ref in zip(one["xs"] + two["xs"], whole["xs"]):
            assert np.array_equal(got, ref)
        np.testing.assert_array_equal((one["rx"] + two["rx"]), whole["rx"])
        np.testing.assert_array_equal((one["re"] + two["re"])[1:], whole["re"][1:])


def test_the_state_between_steps_is_what_the_straight_line_script_holds():
    """S=7, m=1, p=3 stopped after step 2 (middle of the first cycle) and after step 4 (second cycle):
    the state's per-rank samples and caches against the loop-free script of
    test_straight_line_script_S7_m1_p3."""
    f = scalar_predictor
    tau, a, b = O.ddim_coefficients(steps=7)
    st = lambda i, x, e: a[i] * x + b[i] * e
    xT = np.array([0.3, -1.1, 2.0])
    e0 = f(xT, tau[0]);  X1 = st(0, xT, e0)
    E1 = f(X1, tau[1]);  X2 = st(1, X1, E1);  Y2 = st(1, X1, e0);  Z2 = st(1, X1, e0)
    E2 = f(Y2, tau[2]);  X3 = st(2, X2, E2);  Z3 = st(2, Z2, e0)
    E3 = f(Z3, tau[3]);  X4 = st(3, X3, E3)
    E4 = f(X4, tau[4]);  X5 = st(4, X4, E4);  Y5 = st(4, X4, E2);  Z5 = st(4, X4, E3)
    s3 = O.run_sampler(f, xT, tau, a, b, 1, [3, 3], stop=3)["state"]
    assert (s3["step"], s3["cycle"], s3["round"], s3["calls"]) == (3, 0, 2, 3)
    np.testing.assert_allclose(s3["x"][0], X3, rtol=0, atol=1e-12)
    np.testing.assert_allclose(s3["x"][2], Z3, rtol=0, atol=1e-12)      # rank 2 has still to predict
    np.testing.assert_allclose(s3["cache"][1], E2, rtol=0, atol=1e-12)  # rank 1 predicted at step 2
    np.testing.assert_allclose(s3["cache"][2], e0, rtol=0, atol=1e-12)  # rank 2 still holds the warm-up eps
    np.testing.assert_allclose(s3["eps_last"], E2, rtol=0, atol=1e-12)
    s5 = O.run_sampler(f, xT, tau, a, b, 1, [3, 3], stop=5)["state"]
    assert (s5["step"], s5["cycle"], s5["round"], s5["calls"]) == (5, 1, 1, 5)
    for got, ref in zip(s5["x"], [X5, Y5, Z5]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    for got, ref in zip(s5["cache"], [E4, E2, E3]):
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert s5["born"] == [4, 2, 3]
