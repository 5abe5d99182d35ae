"""The forward-only LM-head call that allocates nothing (`dvp_fused_lmhead_forward_noalloc`): its
statistics and partials live in the library's own static device buffer.  Through the C ABI, against
`dvp_fused_lmhead` without grad_out (same logits, sums in another order), on two calls in
a row, the second on a smaller input, with the allocator watched across the calls."""
import ctypes

import pytest
import torch

from paper_2512_23087_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


def _same(a, b, what):
    """Both calls get the same fp32 logits from the same matrix-core kernel, so row maxima, safe-set sizes
    and membership bits are identical; dvp_fused_lmhead sums a row's exponentials in another order (it keeps
    a row block's logits in its workspace and streams over them), so lse and logp agree to fp32 rounding."""
    for k in ("row_max", "safe_count", "safe_bits"):
        x, y = getattr(a, k), getattr(b, k)
        assert (x is None) == (y is None)
        if x is not None:
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), (what, k)
    for k in ("logp", "lse_safe", "lse_full"):
        x, y = getattr(a, k), getattr(b, k)
        assert (x is None) == (y is None)
        if x is not None:
            assert torch.equal(torch.isfinite(x), torch.isfinite(y)), (what, k)
            fin = torch.isfinite(x)
            assert (x[fin] - y[fin]).abs().max().item() <= 1e-5, (what, k)


def _compare(dvp, n, d, v, lr, poison):
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v)
    ref = dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, wl.w_infer, wl.ids, None, lr, lse_full=True, safe_bits=True)
    out_t = dvp.SideOutputs(n, v, "cuda", lse_full=True, safe_bits=True)
    out_i = dvp.SideOutputs(n, v, "cuda", lse_full=True, safe_bits=True)
    flags = torch.empty(n, dtype=torch.uint8, device="cuda")
    for side in (out_t, out_i):                         # stale output contents must not matter
        for k in ("logp", "row_max", "lse_safe", "lse_full"):
            getattr(side, k).fill_(poison)
        side.safe_count.fill_(-7)
        side.safe_bits.fill_(-1)
    flags.fill_(0xFF)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    got = dvp.dvp_fused_lmhead_forward_noalloc(wl.hidden, wl.w_train, wl.w_infer, wl.ids, lr, out_t, out_i, flags)
    after = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    torch.cuda.synchronize()
    assert after == before                              # the binding asked torch for nothing either
    _same(got.train, ref.train, "train")
    _same(got.infer, ref.infer, "infer")
    assert torch.equal(got.row_flags, ref.row_flags)
    assert int(got.train.safe_count.min()) >= 1
    return got


def test_two_calls_in_a_row_the_second_smaller(dvp):
    dvp.prepare()
    lr = dvp.log_rho(1e-4)
    big = _compare(dvp, 700, 256, 5000, lr, poison=3.5)         # several row and column tiles, ragged on both axes
    small = _compare(dvp, 130, 128, 777, lr, poison=-1.25)      # fewer rows, fewer column tiles: stale partials beyond them
    assert big.train.logp.shape[0] == 700 and small.train.logp.shape[0] == 130
    # training side only
    wl = workloads.make_lmhead(device="cuda", n=90, d=64, v=300)
    ref = dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, None, wl.ids, None, lr)
    out_t = dvp.SideOutputs(90, 300, "cuda")
    flags = torch.empty(90, dtype=torch.uint8, device="cuda")
    got = dvp.dvp_fused_lmhead_forward_noalloc(wl.hidden, wl.w_train, None, wl.ids, lr, out_t, None, flags)
    torch.cuda.synchronize()
    _same(got.train, ref.train, "train only")
    assert torch.equal(got.row_flags, ref.row_flags)


def test_sizes_beyond_the_scratch_buffer_are_refused(dvp):
    n, d, v = 16384, 64, 151936          # needs about 234 MB of statistics and partials
    p = dvp.DvpLmHeadParams(n, d, v, d, d, -1.0)
    one = torch.zeros(256, dtype=torch.uint8, device="cuda")    # never dereferenced: the call is refused on the host
    side = dvp.DvpSideOut()
    st = dvp.lib().dvp_fused_lmhead_forward_noalloc(ctypes.byref(p), one.data_ptr(), one.data_ptr(), None,
                                                    one.data_ptr(), ctypes.byref(side), None, None, None)
    assert st == 8 and "scratch" in dvp.status_string(st)
    # the largest row count that fits is accepted by the size check (then stopped by the NULL ids)
    rows = (64 << 20) // (24 * ((v + 255) // 256) + 2048)
    p = dvp.DvpLmHeadParams(rows, d, v, d, d, -1.0)
    st = dvp.lib().dvp_fused_lmhead_forward_noalloc(ctypes.byref(p), one.data_ptr(), one.data_ptr(), None,
                                                    None, ctypes.byref(side), None, None, None)
    assert st == 1
