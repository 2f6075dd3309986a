"""GPU parity of fmt_dls_step (loss-scale controller and denormal-fraction monitor, Sec. II and
Sec. V) against the CPU oracle: every field of the state, after every step, bit for bit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

FIELDS = ("loss_scale", "good_steps", "skip", "steps", "nonfinite", "worst_tensor", "worst_denormal", "worst_total",
          "peak_tensor", "peak_step", "peak_denormal", "peak_total")


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def same_state(fmt, dev_state, ref, what):
    got = fmt.dls_state_to_dict(dev_state)
    want = ref.as_dict()
    for k in FIELDS:
        if k == "loss_scale":
            assert np.float32(got[k]).view(np.uint32) == np.float32(want[k]).view(np.uint32), (what, k, got[k], want[k])
        else:
            assert got[k] == want[k], (what, k, got[k], want[k])


def random_records(rng, count, p_bad):
    h = np.zeros((count, 72), dtype=np.uint64)
    for i in range(count):
        total = int(rng.integers(0, 1 << 20)) if rng.random() < 0.9 else 0
        den = int(rng.integers(0, total + 1)) if rng.random() < 0.7 else 0
        h[i, 0], h[i, 3] = total, den
        if rng.random() < p_bad:
            h[i, 5 + int(rng.integers(0, 3))] = int(rng.integers(1, 1000))
        h[i, 8:] = rng.integers(0, 1000, 64)
    return h


@pytest.mark.parametrize("growth,backoff,interval", [(2.0, 0.5, 3), (1.5, 0.75, 1), (4.0, 0.25, 5), (1.0009765625, 0.9990234375, 2)])
def test_random_sequences(fmt, growth, backoff, interval):
    rng = np.random.default_rng(int(growth * 1000) + interval)
    st = fmt.fmt_dls_init(1024.0)
    ref = oracle.dls_init(1024.0)
    same_state(fmt, st, ref, "init")
    for step in range(80):
        count = int(rng.choice([0, 1, 2, 7, 300, 1000]))
        h = random_records(rng, count, p_bad=0.3 / max(count, 1))
        hd = torch.from_numpy(h.view(np.int64)).cuda() if count else None
        fmt.fmt_dls_step(hd, st, growth=growth, backoff=backoff, interval=interval, min_scale=0.125, max_scale=65536.0)
        oracle.dls_step(h, ref, growth=growth, backoff=backoff, interval=interval, min_scale=0.125, max_scale=65536.0)
        same_state(fmt, st, ref, "step %d" % step)


def test_ties_and_equal_fractions(fmt):
    """Equal fractions in many records (1/2 = 2/4 = ... spread over all lanes of the reduction):
    the lowest index wins, on the device as in the oracle."""
    count = 700
    h = np.zeros((count, 72), dtype=np.uint64)
    for i in range(count):
        h[i, 0], h[i, 3] = 2 * (i % 13 + 1), (i % 13 + 1)
    h[0, 3] = 0                      # the very first record is not among the tied ones
    st = fmt.fmt_dls_step(torch.from_numpy(h.view(np.int64)).cuda(), fmt.fmt_dls_init(2.0))
    ref = oracle.dls_step(h, oracle.dls_init(2.0))
    same_state(fmt, st, ref, "ties")
    assert fmt.dls_state_to_dict(st)["worst_tensor"] == 1


@pytest.mark.parametrize("e,m", [(5, 10), (6, 9)])
def test_training_loop_with_real_statistics(fmt, e, m):
    """Gradient tensors with the spread of config 4 (log2|g| ~ N(-24, 6^2)), scaled by the current
    loss scale, quantized with fused statistics on the GPU; the controller runs on the device from
    those records.  The oracle does the same from its own statistics of the same tensors."""
    rng = np.random.default_rng(5)
    grads = [workloads.log2_normal(n, -24.0, 6.0, 0.01, rng) for n in (4096, 30000, 1000, 65536)]
    st = fmt.fmt_dls_init(2.0 ** 40)
    ref = oracle.dls_init(2.0 ** 40)
    hists = torch.zeros((len(grads), 72), dtype=torch.int64, device="cuda")
    dev = [torch.from_numpy(g).cuda() for g in grads]
    for step in range(40):
        scale = fmt.dls_state_to_dict(st)["loss_scale"]
        assert scale == ref.loss_scale
        rows = []
        for i, g in enumerate(grads):
            scaled = dev[i] * scale                                  # fp32 multiply, as a framework would
            fmt.fmt_quantize(scaled, (e, m, True), hist=hists[i])
            ho = oracle.histogram((g * np.float32(scale)).astype(np.float32), e, m)
            rows.append(np.concatenate([[ho[c] for c in ("total", "zero", "underflow", "denormal", "normal",
                                                           "overflow", "inf", "nan")], ho["bins"]]).astype(np.uint64))
        fmt.fmt_dls_step(hists, st, interval=4, min_scale=1.0, max_scale=2.0 ** 60)
        oracle.dls_step(np.stack(rows), ref, interval=4, min_scale=1.0, max_scale=2.0 ** 60)
        same_state(fmt, st, ref, "step %d" % step)
    final = fmt.dls_state_to_dict(st)
    assert final["steps"] == 40 and final["loss_scale"] < 2.0 ** 40    # the scale did come down
