"""Pins for the oracle's loss-scale controller and denormal-fraction monitor (Sec. II loss scaling
/ dynamic loss scaling; Sec. V highest denormal fraction over all tensors).  The paper states no
update rule; the reading built here is the usual one (halve on a non-finite gradient and skip the
step, double after `interval` clean steps).  It is pinned by a trajectory worked out by hand, by an
independent exact-rational model, and by the closed form of where the scale must settle."""
from fractions import Fraction

import numpy as np

import oracle

N = 72


def rec(total=0, zero=0, underflow=0, denormal=0, normal=0, overflow=0, inf=0, nan=0):
    h = np.zeros(N, dtype=np.uint64)
    h[:8] = [total, zero, underflow, denormal, normal, overflow, inf, nan]
    return h


def test_hand_worked_trajectory():
    """interval 3, start 1024, bounds [256, 4096]; written out by hand."""
    clean = np.stack([rec(total=100, denormal=5, normal=95), rec(total=10, denormal=1, normal=9)])
    ovf = np.stack([rec(total=100, denormal=5, normal=94, overflow=1), rec(total=10, normal=10)])
    inf = np.stack([rec(total=100, normal=100), rec(total=10, normal=8, inf=2)])
    nan = np.stack([rec(total=100, normal=99, nan=1), rec(total=10, normal=10)])
    steps = [clean, clean, clean,      # third clean step doubles: 2048
             clean, ovf,               # run of 1 broken: 1024, skipped
             inf, nan,                 # 512, 256
             nan,                      # clamped at 256
             clean, clean, clean,      # 512
             clean, clean, clean,      # 1024
             clean, clean, clean, clean, clean, clean,   # 2048, 4096
             clean, clean, clean]      # clamped at 4096
    want_scale = [1024, 1024, 2048, 2048, 1024, 512, 256, 256, 256, 256, 512, 512, 512, 1024,
                  1024, 1024, 2048, 2048, 2048, 4096, 4096, 4096, 4096]
    want_skip = [0, 0, 0, 0, 1, 1, 1, 1] + [0] * 15
    want_good = [1, 2, 0, 1, 0, 0, 0, 0, 1, 2, 0, 1, 2, 0, 1, 2, 0, 1, 2, 0, 1, 2, 0]
    st = oracle.dls_init(1024.0)
    for i, h in enumerate(steps):
        oracle.dls_step(h, st, growth=2.0, backoff=0.5, interval=3, min_scale=256.0, max_scale=4096.0)
        assert st.loss_scale == want_scale[i], i
        assert st.skip == want_skip[i], i
        assert st.good_steps == want_good[i], i
        assert st.steps == i + 1
    assert st.nonfinite == 0


def test_nonfinite_is_the_sum_of_three_classes():
    h = np.stack([rec(total=50, normal=40, overflow=3, inf=4, nan=3), rec(total=7, normal=2, overflow=5)])
    st = oracle.dls_step(h, oracle.dls_init(8.0), interval=10)
    assert st.nonfinite == 15 and st.skip == 1 and st.loss_scale == 4.0


def test_worst_tensor_and_running_peak():
    st = oracle.dls_init(1.0)
    a = np.stack([rec(total=100, denormal=10), rec(total=0), rec(total=30, denormal=6), rec(total=10, denormal=2)])
    oracle.dls_step(a, st)
    # 6/30 == 2/10 > 10/100: the tie goes to the lower index; the empty tensor is ignored
    assert (st.worst_tensor, st.worst_denormal, st.worst_total) == (2, 6, 30)
    assert (st.peak_tensor, st.peak_step, st.peak_denormal, st.peak_total) == (2, 0, 6, 30)
    b = np.stack([rec(total=100, denormal=20), rec(total=5, denormal=1), rec(total=30), rec(total=10)])
    oracle.dls_step(b, st)
    # equal to the peak (1/5): the peak is only replaced by a strictly larger fraction
    assert (st.worst_tensor, st.worst_denormal, st.worst_total) == (0, 20, 100)
    assert (st.peak_tensor, st.peak_step) == (2, 0)
    c = np.stack([rec(total=100), rec(total=3, denormal=1)])
    oracle.dls_step(c, st)
    assert (st.peak_tensor, st.peak_step, st.peak_denormal, st.peak_total) == (1, 2, 1, 3)
    oracle.dls_step(np.zeros((0, N), dtype=np.uint64), st)        # a step without tensors
    assert st.worst_tensor == -1 and st.peak_step == 2 and st.skip == 0 and st.steps == 4


def model_step(state, hists, growth, backoff, interval, lo, hi):
    """The same controller with exact rationals and Python floats narrowed to fp32 by numpy."""
    nonfinite = sum(int(h[5]) + int(h[6]) + int(h[7]) for h in hists)
    best, best_frac = -1, None
    for i, h in enumerate(hists):
        if int(h[0]) > 0:
            f = Fraction(int(h[3]), int(h[0]))
            if best_frac is None or f > best_frac:
                best, best_frac = i, f
    s = np.float32(state["scale"])
    if nonfinite:
        s = max(np.float32(s * np.float32(backoff)), np.float32(lo))
        state["good"] = 0
    else:
        state["good"] += 1
        if state["good"] >= interval:
            s = min(np.float32(s * np.float32(growth)), np.float32(hi))
            state["good"] = 0
    state["scale"] = float(s)
    state["skip"] = int(nonfinite > 0)
    if best >= 0 and (state["peak"] is None or best_frac > state["peak"][0]):
        state["peak"] = (best_frac, best, state["steps"])
    state["worst"] = best
    state["steps"] += 1
    return state


def test_against_exact_rational_model():
    rng = np.random.default_rng(11)
    for trial in range(20):
        growth, backoff = [(2.0, 0.5), (1.5, 0.75), (4.0, 0.25), (1.0009765625, 0.9990234375)][trial % 4]
        interval = int(rng.integers(1, 6))
        st = oracle.dls_init(64.0)
        ms = {"scale": 64.0, "good": 0, "steps": 0, "peak": None, "skip": 0, "worst": -1}
        for step in range(60):
            count = int(rng.integers(0, 6))
            h = np.zeros((count, N), dtype=np.uint64)
            for i in range(count):
                total = int(rng.integers(0, 50))
                den = int(rng.integers(0, total + 1))
                bad = int(rng.random() < 0.1) * int(rng.integers(1, 4))
                h[i, 0], h[i, 3] = total, den
                h[i, 5 + int(rng.integers(0, 3))] = bad
            oracle.dls_step(h, st, growth=growth, backoff=backoff, interval=interval, min_scale=0.5, max_scale=4096.0)
            model_step(ms, h, growth, backoff, interval, 0.5, 4096.0)
            assert st.loss_scale == np.float32(ms["scale"]) and st.skip == ms["skip"] and st.good_steps == ms["good"]
            assert st.worst_tensor == ms["worst"]
            if ms["peak"] is not None:
                assert (st.peak_tensor, st.peak_step) == ms["peak"][1:]
                assert Fraction(int(st.peak_denormal), int(st.peak_total)) == ms["peak"][0]


def test_scale_settles_at_the_closed_form():
    """A fixed gradient tensor, statistics of S*g from the oracle's own histogram: from a scale that
    overflows the controller must halve down to the largest power of two that keeps S*max|g| below
    the overflow threshold of the format, then cycle: `interval` clean steps, one doubling that
    overflows, one halving."""
    e, m = 5, 10
    rng = np.random.default_rng(3)
    g = (rng.standard_normal(4096) * 2.0 ** -12).astype(np.float32)
    gmax = float(np.max(np.abs(g)))
    ovf = (2.0 - 2.0 ** -(m + 1)) * 2.0 ** 15                     # first magnitude that rounds to infinity
    k = int(np.floor(np.log2(ovf / gmax)))
    while gmax * 2.0 ** k >= ovf:
        k -= 1
    best = 2.0 ** k                                              # largest safe power of two
    st = oracle.dls_init(2.0 ** 30)
    scales = []
    for step in range(40):
        h = oracle.histogram((g.astype(np.float64) * st.loss_scale).astype(np.float32), e, m)
        rec_ = np.concatenate([[h[c] for c in ("total", "zero", "underflow", "denormal", "normal", "overflow", "inf", "nan")],
                               h["bins"]]).astype(np.uint64)
        oracle.dls_step(rec_[None, :], st, interval=4, min_scale=1.0, max_scale=2.0 ** 40)
        scales.append(st.loss_scale)
    down = 30 - k                                                 # halvings needed from 2^30
    assert scales[:down] == [2.0 ** (29 - i) for i in range(down)]
    tail = scales[down:]
    # 3 clean steps at `best`, the 4th doubles, the next overflows and halves again
    period = [best, best, best, 2 * best, best]
    for i, s in enumerate(tail):
        assert s == period[i % 5], (i, s)
