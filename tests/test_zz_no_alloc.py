"""fmt_quantize_static, the entry point that allocates nothing: its partial statistics records live in
a file-scope device array of the library instead of scratch created with hipMalloc.  Called through the
raw C ABI and compared bit for bit -- rounded values and all 72 counts -- with fmt_quantize on the same
inputs: two calls in a row on one GPU, the second on a smaller tensor (the array keeps the first
call's contents), then against the CPU oracle."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads

torch = pytest.importorskip("torch")


def test_static_entry_validates_before_touching_the_gpu():
    import paper_2103_15940_amd as fmt
    lib = fmt.raw_library()
    f = fmt._CFormat(6, 9, 1)
    buf = (ctypes.c_float * 8)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    too_many = (1 << 36) + 1
    assert lib.fmt_quantize_static(p, p, too_many, f, None, -48, None) == -3          # beyond the stated maximum
    assert lib.fmt_quantize_static(None, p, 4, f, None, -48, None) == -2
    assert lib.fmt_quantize_static(p, p, 4, fmt._CFormat(9, 9, 1), None, -48, None) == -1
    assert lib.fmt_quantize_static(p.value + 2, p, 1, f, None, -48, None) == -4
    assert lib.fmt_quantize_static(p, p.value + 4, 4, f, None, -48, None) == -6         # partial overlap
    assert lib.fmt_quantize_static(p, p, 4, f, p, 500, None) == -5                      # exp_lo outside its range
    assert lib.fmt_quantize_static(None, None, 0, f, None, -48, None) == 0              # empty, no statistics: nothing to do


@pytest.mark.gpu
def test_static_entry_matches_fmt_quantize_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as fmt
    lib = fmt.raw_library()
    dev = torch.device("cuda")
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(2103)
    # several tiles and a ragged tail, then a smaller tensor; special values in both
    sizes = [5 * 4096 * 16 + 1237, 4096 + 19]
    for call, n in enumerate(sizes):
        for (e, m, d) in [(6, 9, True), (5, 10, False), (8, 7, True)]:
            x_host = np.concatenate([workloads.log2_normal(n - 28, -14.0, 7.0, 0.02, rng), workloads.special_values()])
            x = torch.from_numpy(x_host).to(dev)
            y_static, y_plain = torch.empty_like(x), torch.empty_like(x)
            h_static, h_plain = fmt.new_hist(dev), fmt.new_hist(dev)
            h_static.fill_(-1)
            rc = lib.fmt_quantize_static(x.data_ptr(), y_static.data_ptr(), n, fmt._CFormat(e, m, int(d)),
                                         h_static.data_ptr(), -48, stream)
            assert rc == 0, fmt.status_string(rc)
            fmt.fmt_quantize(x, (e, m, d), out=y_plain, hist=h_plain)
            torch.cuda.synchronize()
            assert torch.equal(y_static.view(torch.int32), y_plain.view(torch.int32)), (call, n, e, m, d)
            assert torch.equal(h_static, h_plain), (call, n, e, m, d)
            want = oracle.quantize(x_host, e, m, d)
            assert np.array_equal(y_static.cpu().numpy().view(np.uint32), want.view(np.uint32))
            got, ho = fmt.hist_to_dict(h_static), oracle.histogram(x_host, e, m)
            assert all(got[k] == ho[k] for k in fmt.CLASS_NAMES) and np.array_equal(got["bins"], ho["bins"])
    # without statistics the array is not touched; in place; an empty tensor with statistics gives zeros
    x = torch.from_numpy(workloads.log2_normal(1000, -14.0, 6.0, 0.0, rng)).to(dev)
    want = fmt.fmt_quantize(x, (6, 9, True))
    assert lib.fmt_quantize_static(x.data_ptr(), x.data_ptr(), 1000, fmt._CFormat(6, 9, 1), None, -48, stream) == 0
    h = fmt.new_hist(dev)
    h.fill_(7)
    assert lib.fmt_quantize_static(None, None, 0, fmt._CFormat(6, 9, 1), h.data_ptr(), -48, stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(x, want) and int(h.abs().sum()) == 0
