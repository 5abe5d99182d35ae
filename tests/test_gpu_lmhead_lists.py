"""GPU parity of dvp_fused_lmhead_lists (the LM-head variant with the gradient kept as per-row lists)
against the fp64 oracle, through the C ABI.

Forward outputs: the bars of tests/test_gpu_lmhead.py (the same two GEMM passes produce them).
Gradient: nothing passes through bf16 here, so what separates the GPU from the oracle is the fp32
accumulation of the logits and of the sums.  A logit is accumulated over d / 16 matrix-instruction steps,
each rounding a partial sum of magnitude up to max|z| to fp32: half a unit in the last place per step,
adding up like a random walk, is sqrt(d / 16) 2^-24 max|z| (2^-20 max|z| at d = 4096); the bound used is twice
that at the largest d, dz = 2^-19 (max|z| + 10), and it moves a probability by at most 2 p dz to first
order.  Per element
    |dH_gpu - dH| <= 2 dz (|c| p) |W| + 1e-5 + 2^-20 |dH|,   |dW_gpu - dW| <= 2 dz (|c| p)^T |H| + 1e-5 + 2^-20 |dW|,
and a list value is within 2 dz |c| p_k + 1e-6 of the oracle's dz.  Rows with a logit inside the band
around the threshold (membership may differ between fp32 and fp64 logits) are given grad_out = 0 on both
sides, so they drop out of dH and dW; their forward outputs are still compared, band-aware.
Rows whose safe set is longer than the list are flagged and contribute nothing: the oracle is given
grad_out = 0 for them.
"""
import numpy as np
import pytest
import torch

from oracle import dvp_oracle as orc
from paper_2512_23087_amd import workloads
from tests.test_gpu_lmhead import BAND, _check_side

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


def _run(dvp, wl, rho, cap, infer=True, lse_full=False, abs_check=True):
    lr = dvp.log_rho(rho)
    ids = wl.ids.cpu().numpy()
    n = ids.shape[0]
    H, Wt, Wi = wl.hidden.cpu(), wl.w_train.cpu(), wl.w_infer.cpu()
    fwd = orc.lmhead(H, Wt, ids, np.float32(lr), band=BAND, want_flags=True, threads=8)
    band_rows = fwd["band_count"] > 0
    g = wl.grad_out.cpu().numpy().astype(np.float64).copy()
    g[band_rows] = 0.0
    gout = torch.tensor(g, dtype=torch.float32, device="cuda")
    res = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, wl.w_infer if infer else None, wl.ids, gout, lr, cap,
                                     lse_full=lse_full)
    torch.cuda.synchronize()

    same_t = _check_side("train", res.train, fwd, fwd)
    flags = res.row_flags.cpu().numpy()
    np.testing.assert_array_equal((flags & 1)[same_t], fwd["y_in_safe"][same_t])
    if infer:
        oi = orc.lmhead(H, Wi, ids, np.float32(lr), band=BAND, threads=8)
        same_i = _check_side("infer", res.infer, oi, oi)
        np.testing.assert_array_equal(((flags >> 1) & 1)[same_i], oi["y_in_safe"][same_i])
    else:
        assert res.infer is None and not (flags & 2).any()

    clean = ~band_rows
    y_safe = fwd["y_in_safe"] == 1
    over = y_safe & (fwd["safe_count"] > cap)
    np.testing.assert_array_equal(((flags & dvp.ROW_GRAD_OVERFLOW) != 0)[clean], over[clean])
    glen = res.grad_len.cpu().numpy()
    np.testing.assert_array_equal(glen[clean], np.where(y_safe, fwd["safe_count"], 0)[clean])

    g_eff = g.copy()
    g_eff[over] = 0.0
    ot = orc.lmhead(H, Wt, ids, np.float32(lr), grad_out=g_eff, band=BAND, threads=8)
    dz_round = 2.0 ** -19 * (np.abs(ot["row_max"]).max() + 10.0)
    listed = clean & y_safe & ~over
    for i in np.nonzero(listed)[0]:
        idx, val = res.row(int(i))
        want = np.nonzero(fwd["safe_flags"][i])[0]
        np.testing.assert_array_equal(idx.numpy(), want)
        stored = res.entries[i, :len(want), 0].cpu().numpy().astype(np.int64) & 0xFFFFFFFF
        np.testing.assert_array_equal(stored, want)                      # sorted by token on the device
        ref = ot["dz"][i, want]
        pk = np.abs(ref).copy()
        pk[want == ids[i]] = abs(g[i]) * np.exp(ot["logp"][i])
        assert np.all(np.abs(val.double().numpy() - ref) <= 2 * dz_round * pk + 1e-6 * max(1.0, abs(g[i])))
    full = np.abs(ot["dz"])
    rows = np.nonzero(listed)[0]
    full[rows, ids[rows]] = np.abs(g[rows]) * np.exp(ot["logp"][rows])
    H64, W64 = H.double().numpy(), Wt.double().numpy()
    bound_h = 2 * dz_round * (full @ np.abs(W64)) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_hidden"])
    bound_w = 2 * dz_round * (full.T @ np.abs(H64)) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_w"])
    dh = res.d_hidden.cpu().double().numpy()
    dw = res.d_w.cpu().double().numpy()
    err_h = (np.abs(dh - ot["d_hidden"]) / bound_h).max()
    err_w = (np.abs(dw - ot["d_w"]) / bound_w).max()
    print("cap %d: %d listed rows, %d overflow, %d band; dH at %.3f, dW at %.3f of their bounds" %
          (cap, listed.sum(), (over & clean).sum(), band_rows.sum(), err_h, err_w))
    assert err_h <= 1.0 and err_w <= 1.0
    if abs_check:   # the bf16-input bar, where the gradients are O(1)
        assert np.abs(dh - ot["d_hidden"]).max() <= 2e-3 and np.abs(dw - ot["d_w"]).max() <= 2e-3
    assert np.all(dh[~listed] == 0.0)
    return res, fwd, listed


def test_peaked_rows_against_oracle(dvp):
    """Short safe sets: each side's forward is finished from the candidates of its first pass; with
    lse_full every token's exponential is needed and the second pass runs instead."""
    wl = workloads.make_lmhead(device="cuda", n=300, d=128, v=3000, hidden_scale=60.0)
    for rho, cap in ((1e-4, 64), (1e-2, 16), (1e-4, 8)):
        res, fwd, listed = _run(dvp, wl, rho, cap)
        assert listed.sum() > 50
        assert res.second_pass.tolist() == [0, 0]          # one pass over the logits per side was enough
    assert np.median(fwd["safe_count"]) < 64
    _run(dvp, wl, 1e-4, 64, lse_full=True)


def test_flat_rows_among_peaked_ones(dvp):
    """A few rows with tiny hidden states (flat logits: every token is a candidate, more than are kept)
    go through the second pass, gathered; the peaked rows are finished from their candidates."""
    wl = workloads.make_lmhead(device="cuda", n=520, d=128, v=3000, hidden_scale=60.0)
    wl.hidden[::37] = (wl.hidden[::37].float() * 1e-3).to(torch.bfloat16)
    res, fwd, listed = _run(dvp, wl, 1e-4, 64)
    assert (fwd["safe_count"][::37] == 3000).all() and listed.sum() > 300
    assert res.second_pass.tolist() == [len(range(0, 520, 37))] * 2    # exactly the flat rows, on both sides
    # and a row whose sampled token is far below the maximum: no help from it for the bound
    wl = workloads.make_lmhead(device="cuda", n=300, d=128, v=900, hidden_scale=60.0)
    z = wl.hidden.float() @ wl.w_train.float().T
    wl.ids[:50] = z[:50].argmin(dim=1)
    res, fwd, listed = _run(dvp, wl, 1e-4, 64)
    assert (fwd["y_in_safe"][:50] == 0).all() and (res.grad_len[:50] == 0).all()
    assert res.second_pass.tolist() == [0, 0]              # 900 tokens: whatever the bound, the candidates fit


def test_large_magnitude_hidden_states_never_break_the_sampled_token_bound(dvp):
    """The one-pass route collects candidates above a bound built to lie below the sampled token's logit as
    the matrix cores deliver it; a row where it did not would be sent through the second pass.  With logits
    in the hundreds (hidden states x 100 and x 250) no row is: the second-pass counters stay at zero and
    every output still matches the oracle."""
    for scale, d in ((100.0, 512), (250.0, 128)):
        wl = workloads.make_lmhead(device="cuda", n=300, d=d, v=3000, hidden_scale=scale)
        res, fwd, listed = _run(dvp, wl, 1e-4, 64, abs_check=False)
        assert np.abs(fwd["row_max"]).max() > 100.0
        assert res.second_pass.tolist() == [0, 0]
        assert listed.sum() > 100


@pytest.mark.parametrize("n,d,v,cap", [(1, 64, 3, 4), (2, 64, 1, 1), (257, 192, 257, 300), (33, 64, 513, 1024),
                                       (700, 64, 900, 1000), (300, 64, 1500, 1000)])
def test_shapes_and_long_lists(dvp, n, d, v, cap):
    # flat logits: every token is safe, lists as long as the vocabulary (or overflowing), several row blocks
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v)
    _run(dvp, wl, 1e-2, cap)
    _run(dvp, wl, 0.0, cap, infer=False)


def test_agrees_with_the_dense_call_and_repeats_bit_for_bit(dvp):
    wl = workloads.make_lmhead(device="cuda", n=1000, d=256, v=5000, hidden_scale=40.0)
    lr = dvp.log_rho(1e-4)
    a = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, 1024)
    b = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, 1024)
    ref = dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr)
    torch.cuda.synchronize()
    assert not (a.row_flags & dvp.ROW_GRAD_OVERFLOW).any()
    valid = torch.arange(1024, device="cuda")[None, :] < a.grad_len[:, None]     # entries past a row's length are unspecified
    for x, y in ((a.d_hidden, b.d_hidden), (a.d_w, b.d_w), (a.entries[valid], b.entries[valid]), (a.grad_len, b.grad_len)):
        assert torch.equal(x, y)
    assert torch.equal(a.train.logp, b.train.logp) and torch.equal(a.infer.lse_safe, b.infer.lse_safe)
    # the same logits, thresholds and safe sets as the dense call; the sums run in another order (by token
    # here, by tile there); the dense call rounds E to bf16, so gradients agree to 2^-8 relative
    assert torch.equal(a.train.row_max, ref.train.row_max) and torch.equal(a.infer.row_max, ref.infer.row_max)
    assert torch.equal(a.train.safe_count, ref.train.safe_count) and torch.equal(a.row_flags, ref.row_flags)
    for x, y in ((a.train.logp, ref.train.logp), (a.infer.logp, ref.infer.logp), (a.train.lse_safe, ref.train.lse_safe)):
        fin = torch.isfinite(y)
        assert torch.equal(torch.isfinite(x), fin) and (x[fin] - y[fin]).abs().max().item() <= 2e-6 * (1 + y[fin].abs().max().item())
    scale_h = ref.d_hidden.abs().max().item()
    scale_w = ref.d_w.abs().max().item()
    assert (a.d_hidden - ref.d_hidden).abs().max().item() <= 2.0 ** -6 * scale_h
    assert (a.d_w - ref.d_w).abs().max().item() <= 2.0 ** -6 * scale_w


def test_forward_only(dvp):
    """Without grad_out the call is the forward of both sides: one pass per side over peaked rows, a
    gathered second pass for the flat ones."""
    wl = workloads.make_lmhead(device="cuda", n=520, d=128, v=3000, hidden_scale=60.0)
    wl.hidden[::41] = (wl.hidden[::41].float() * 1e-3).to(torch.bfloat16)
    lr = dvp.log_rho(1e-4)
    res = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, wl.w_infer, wl.ids, None, lr, 64)
    torch.cuda.synchronize()
    assert res.d_hidden is None and res.entries is None
    assert res.second_pass.tolist() == [len(range(0, 520, 41))] * 2
    ids = wl.ids.cpu().numpy()
    H = wl.hidden.cpu()
    ot = orc.lmhead(H, wl.w_train.cpu(), ids, np.float32(lr), band=BAND, threads=8)
    oi = orc.lmhead(H, wl.w_infer.cpu(), ids, np.float32(lr), band=BAND, threads=8)
    same_t = _check_side("train", res.train, ot, ot)
    same_i = _check_side("infer", res.infer, oi, oi)
    flags = res.row_flags.cpu().numpy()
    np.testing.assert_array_equal((flags & 1)[same_t], ot["y_in_safe"][same_t])
    np.testing.assert_array_equal(((flags >> 1) & 1)[same_i], oi["y_in_safe"][same_i])
    assert not (flags & 0xFC).any()


def test_8bit_inference_engine(dvp):
    """The inference side as an E4M3 engine (activations, head and a scale): checked against the oracle's
    logits from the codes; the training side, the lists and the gradient do not depend on it.
    Peaked rows need logits of +-40 here, which the engine forms from products of up to 448 x 448 summed in
    fp32 before the scale: their accumulation rounding reaches 8e-4 (2e-5 relative), so the membership band
    and the row-maximum bar are 2e-3, the absolute tolerance of low-precision inputs, instead of 2e-4."""
    wl = workloads.make_lmhead(device="cuda", n=520, d=256, v=3000, hidden_scale=40.0, f8_engine=True)
    wl.hidden[::53] = (wl.hidden[::53].float() * 1e-3).to(torch.bfloat16)          # flat training rows
    wl.hidden8.view(torch.uint8)[::47] = 0                                         # flat inference rows (all logits 0)
    lr = dvp.log_rho(1e-4)
    res = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, 64,
                                     infer_f8=(wl.hidden8, wl.w8, wl.scale_infer))
    ref = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, 64)
    torch.cuda.synchronize()
    assert res.second_pass.tolist() == [len(range(0, 520, 53)), len(range(0, 520, 47))]
    ids = wl.ids.cpu().numpy()
    h8 = wl.hidden8.view(torch.uint8).cpu().numpy()
    w8 = wl.w8.view(torch.uint8).cpu().numpy()
    oi = orc.lmhead(h8, w8, ids, np.float32(lr), band=2e-3, threads=8, scale=wl.scale_infer)
    same_i = _check_side("infer", res.infer, oi, oi, band=2e-3)
    flags = res.row_flags.cpu().numpy()
    np.testing.assert_array_equal(((flags >> 1) & 1)[same_i], oi["y_in_safe"][same_i])
    assert (oi["safe_count"][::47] == 3000).all() and (oi["band_count"] == 0).mean() > 0.9
    for k in ("logp", "row_max", "lse_safe", "safe_count"):
        assert torch.equal(getattr(res.train, k), getattr(ref.train, k)), k
    assert torch.equal(res.row_flags & 13, ref.row_flags & 13)
    assert torch.equal(res.d_hidden, ref.d_hidden) and torch.equal(res.d_w, ref.d_w)
    assert torch.equal(res.grad_len, ref.grad_len)
    # with lse_full both sides run both passes over all rows (every token's exponential is needed)
    full = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, 64, lse_full=True,
                                      infer_f8=(wl.hidden8, wl.w8, wl.scale_infer))
    torch.cuda.synchronize()
    assert full.second_pass.tolist() == [0, 0]
    _check_side("infer", full.infer, oi, oi, band=2e-3)
    assert torch.equal(full.infer.safe_count, res.infer.safe_count) and torch.equal(full.row_flags, res.row_flags)
    assert torch.equal(full.grad_len, res.grad_len)
    assert (full.d_w - res.d_w).abs().max().item() <= 1e-5 * (1 + res.d_w.abs().max().item())


def test_padded_strides_and_out_of_range_ids(dvp):
    """Row strides larger than the hidden size (NaN in the padding) and sampled ids outside [0, V):
    flagged per row, NaN log-probs, an empty list, nothing else disturbed."""
    n, d, v, pad = 300, 128, 3000, 8
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v, hidden_scale=60.0)
    H = torch.full((n, d + pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    W = torch.full((v, d + pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    H[:, :d] = wl.hidden
    W[:, :d] = wl.w_train
    ids = wl.ids.clone()
    ids[3] = -1
    ids[77] = v
    lr = dvp.log_rho(1e-4)
    a = dvp.dvp_fused_lmhead_lists(H[:, :d], W[:, :d], None, ids, wl.grad_out, lr, 64)
    torch.cuda.synchronize()
    flags = a.row_flags.cpu().numpy()
    assert flags[3] == 4 and flags[77] == 4 and (np.delete(flags, [3, 77]) & 4).sum() == 0
    assert torch.isnan(a.train.logp[3]) and torch.isnan(a.train.logp[77])
    assert a.grad_len[3] == 0 and a.grad_len[77] == 0
    assert torch.all(a.d_hidden[3] == 0) and torch.all(a.d_hidden[77] == 0)
    assert torch.isfinite(a.d_w).all() and torch.isfinite(a.d_hidden).all()
    assert a.d_hidden.stride(0) == d + pad and a.d_w.stride(0) == d + pad
    g2 = wl.grad_out.clone()
    g2[3] = 0
    g2[77] = 0
    ids2 = ids.clone()
    ids2[3] = 0
    ids2[77] = 0
    b = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, ids2, g2, lr, 64)
    torch.cuda.synchronize()
    keep = torch.ones(n, dtype=torch.bool, device="cuda")
    keep[3] = keep[77] = False
    assert torch.equal(a.train.logp[keep], b.train.logp[keep]) and torch.equal(a.train.safe_count, b.train.safe_count)
    assert torch.equal(a.d_hidden[keep], b.d_hidden[keep]) and torch.equal(a.d_w, b.d_w)


def test_lists_then_dense_rows_give_the_whole_gradient(dvp):
    """Peaked rows with flat ones among them: the list form covers the rows whose safe set fits the list,
    dvp_fused_lmhead_rows adds the dense gradient of the flagged ones.  Together: the gradient of every
    row, against the oracle with the dense call's per-element bounds (the flagged rows' entries pass
    through bf16 there) and against the dense call itself."""
    n, d, v, cap = 520, 128, 3000, 64
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v, hidden_scale=60.0)
    wl.hidden[::13] = (wl.hidden[::13].float() * 0.05).to(torch.bfloat16)          # wide rows: hundreds of safe tokens
    lr = dvp.log_rho(1e-4)
    ids = wl.ids.cpu().numpy()
    H, Wt = wl.hidden.cpu(), wl.w_train.cpu()
    fwd = orc.lmhead(H, Wt, ids, np.float32(lr), band=BAND, threads=8)
    g = wl.grad_out.cpu().numpy().astype(np.float64).copy()
    g[fwd["band_count"] > 0] = 0.0
    gout = torch.tensor(g, dtype=torch.float32, device="cuda")
    res = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, gout, lr, cap)
    torch.cuda.synchronize()
    over = torch.nonzero((res.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).squeeze(1).to(torch.int32)
    assert 20 <= over.numel() <= 60
    # an index out of range among them is skipped
    rows = torch.cat([over, torch.tensor([-1, n], dtype=torch.int32, device="cuda")])
    dvp.dvp_fused_lmhead_rows(wl.hidden, wl.w_train, wl.ids, gout, lr, rows, res.d_hidden, res.d_w)
    torch.cuda.synchronize()
    ot = orc.lmhead(H, Wt, ids, np.float32(lr), grad_out=g, band=BAND, threads=8)
    H64, W64 = H.double().numpy(), Wt.double().numpy()
    dense_rows = np.zeros(n, bool)
    dense_rows[over.cpu().numpy()] = True
    soft = np.abs(ot["dz"]) * dense_rows[:, None]           # the entries that went through bf16
    safe_rows = np.nonzero(ot["y_in_safe"])[0]
    soft[safe_rows, ids[safe_rows]] = 0.0
    full = np.abs(ot["dz"])
    full[safe_rows, ids[safe_rows]] = np.abs(g[safe_rows]) * np.exp(ot["logp"][safe_rows])
    dz_round = 2.0 ** -19 * (np.abs(ot["row_max"]).max() + 10.0)
    bound_h = 2.0 ** -8 * (soft @ np.abs(W64)) + 2 * dz_round * (full @ np.abs(W64)) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_hidden"])
    bound_w = 2.0 ** -7 * (soft.T @ np.abs(H64)) + 2 * dz_round * (full.T @ np.abs(H64)) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_w"])
    dh = res.d_hidden.cpu().double().numpy()
    dw = res.d_w.cpu().double().numpy()
    err_h, err_w = (np.abs(dh - ot["d_hidden"]) / bound_h).max(), (np.abs(dw - ot["d_w"]) / bound_w).max()
    print("dH at %.3f, dW at %.3f of their bounds (%d rows dense)" % (err_h, err_w, over.numel()))
    assert err_h <= 1.0 and err_w <= 1.0
    assert np.abs(dh - ot["d_hidden"]).max() <= 2e-3 and np.abs(dw - ot["d_w"]).max() <= 2e-3
    assert np.abs(ot["d_hidden"][dense_rows]).max() > 0


def test_flagged_rows_chosen_and_counted_on_the_device(dvp):
    """The same two steps with no read-back: dvp_fused_lmhead_select_rows lists the flagged rows and counts them
    on the device, dvp_fused_lmhead_rows_counted sizes its launches for an upper bound and finds the count
    there.  Results are identical to the host-counted call, for a bound well above the count, for a bound
    equal to it, for inputs without a flagged row, and for more than one row block's worth of bound."""
    n, d, v, cap = 520, 128, 3000, 64
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v, hidden_scale=60.0)
    peaked = wl.hidden.clone()
    wl.hidden[::13] = (wl.hidden[::13].float() * 0.05).to(torch.bfloat16)
    lr = dvp.log_rho(1e-4)

    def lists(hidden):
        r = dvp.dvp_fused_lmhead_lists(hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, cap)
        torch.cuda.synchronize()
        return r

    ref = lists(wl.hidden)
    over = torch.nonzero((ref.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).squeeze(1).to(torch.int32)
    dvp.dvp_fused_lmhead_rows(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, over, ref.d_hidden, ref.d_w)
    torch.cuda.synchronize()
    for max_rows in (over.numel(), 100, 300):
        res = lists(wl.hidden)
        rows = torch.full((max_rows,), 12345, dtype=torch.int32, device="cuda")
        n_sub = torch.full((1,), -5, dtype=torch.int32, device="cuda")
        n_flag = torch.full((1,), -5, dtype=torch.int32, device="cuda")
        dvp.dvp_fused_lmhead_select_rows(res.row_flags, dvp.ROW_GRAD_OVERFLOW, rows, n_sub, n_flagged=n_flag)
        dvp.dvp_fused_lmhead_rows_counted(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, rows, n_sub, res.d_hidden, res.d_w)
        torch.cuda.synchronize()
        assert n_sub.item() == over.numel() == n_flag.item()
        assert torch.equal(rows[:over.numel()], over) and torch.all(rows[over.numel():] == -1)
        assert torch.equal(res.d_hidden, ref.d_hidden) and torch.equal(res.d_w, ref.d_w), max_rows
    # a bound below the count: the first rows only, and the true count is still reported
    rows = torch.empty(7, dtype=torch.int32, device="cuda")
    dvp.dvp_fused_lmhead_select_rows(ref.row_flags, dvp.ROW_GRAD_OVERFLOW, rows, n_sub, n_flagged=n_flag)
    torch.cuda.synchronize()
    assert n_sub.item() == 7 and n_flag.item() == over.numel() and torch.equal(rows, over[:7])
    # no flagged row: the counted call changes nothing
    res = lists(peaked)
    assert not ((res.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).any()
    dh0, dw0 = res.d_hidden.clone(), res.d_w.clone()
    rows = torch.empty(64, dtype=torch.int32, device="cuda")
    dvp.dvp_fused_lmhead_select_rows(res.row_flags, dvp.ROW_GRAD_OVERFLOW, rows, n_sub)
    dvp.dvp_fused_lmhead_rows_counted(peaked, wl.w_train, wl.ids, wl.grad_out, lr, rows, n_sub, res.d_hidden, res.d_w)
    torch.cuda.synchronize()
    assert n_sub.item() == 0 and torch.equal(res.d_hidden, dh0) and torch.equal(res.d_w, dw0)


def test_flagged_rows_beyond_one_row_block(dvp):
    """An upper bound of more than 8192 rows (two row blocks of the dense call), the count inside the first
    block or reaching into the second: identical to the host-counted call."""
    n, d, v = 9000, 64, 700
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v)
    lr = dvp.log_rho(1e-4)
    for count in (300, 8400):
        flags = torch.zeros(n, dtype=torch.uint8, device="cuda")
        pick = torch.randperm(n, device="cuda", generator=torch.Generator(device="cuda").manual_seed(count))[:count]
        flags[pick] = 8
        chosen = torch.nonzero(flags != 0).squeeze(1).to(torch.int32)
        dh_ref = torch.zeros(n, d, device="cuda")
        dw_ref = torch.zeros(v, d, device="cuda")
        dvp.dvp_fused_lmhead_rows(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, chosen, dh_ref, dw_ref)
        dh, dw = torch.zeros(n, d, device="cuda"), torch.zeros(v, d, device="cuda")
        rows = torch.empty(n, dtype=torch.int32, device="cuda")
        n_sub = torch.zeros(1, dtype=torch.int32, device="cuda")
        dvp.dvp_fused_lmhead_select_rows(flags, 8, rows, n_sub)
        dvp.dvp_fused_lmhead_rows_counted(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, rows, n_sub, dh, dw)
        torch.cuda.synchronize()
        assert n_sub.item() == count
        assert torch.equal(dh, dh_ref) and torch.equal(dw, dw_ref), count
        assert dh_ref.abs().max().item() > 0


def test_many_rows(dvp):
    """100,000 token rows of a small head: 256 row blocks of 391 rows in the column-major copy, several
    rows per thread in the compaction of the second-pass rows."""
    wl = workloads.make_lmhead(device="cuda", n=100000, d=64, v=2500, hidden_scale=150.0)
    wl.hidden[::997] = (wl.hidden[::997].float() * 1e-3).to(torch.bfloat16)
    # dW sums 100,000 rows of hidden states of magnitude 150: entries reach 500, so only the per-element
    # bound (relative 2^-20 and up) is meaningful, not the absolute figure
    res, fwd, listed = _run(dvp, wl, 1e-4, 32, abs_check=False)
    assert res.second_pass.tolist() == [len(range(0, 100000, 997))] * 2
    assert listed.sum() > 50000


def test_validation(dvp):
    wl = workloads.make_lmhead(device="cuda", n=16, d=64, v=100)
    lr = dvp.log_rho(1e-2)
    for cap, status in ((0, 3), (1025, 5)):
        with pytest.raises(dvp.DvpError) as e:
            dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, cap,
                                       workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
        assert e.value.status == status
    with pytest.raises(dvp.DvpError) as e:
        dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, 8,
                                   workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 6


def test_full_size_peaked_sampled_rows(dvp):
    """configs[4]'s shape (N=16384, d=4096, V=151936) with the hidden states scaled by 20 (a few safe
    tokens per row), list_cap 64, as the benchmark runs it: forward outputs, list entries and dH on sampled
    rows against the oracle.  dW[k, :] needs every row's statistics, so at this size it is checked through
    properties: its columns sum to zero (each row's dz does, Prop. 5.4); rows of tokens that no list holds
    are exactly zero; and it equals the lists' own transpose product formed in fp64 by torch (the lists
    being checked against the oracle on the sampled rows): that covers the column-major copy at full size."""
    wl = workloads.make_lmhead(device="cuda", hidden_scale=20.0)
    n, d = wl.hidden.shape
    v = wl.w_train.shape[0]
    cap = 64
    lr = dvp.log_rho(1e-4)
    res = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, cap)
    torch.cuda.synchronize()
    assert res.second_pass.tolist() == [0, 0]
    rng = np.random.default_rng(2)
    rows = np.unique(np.concatenate([[0, n - 1], rng.choice(n, 46, replace=False)]))
    ridx = torch.as_tensor(rows, device="cuda")
    H = wl.hidden[ridx].cpu()
    ids = wl.ids[ridx].cpu().numpy()
    g = wl.grad_out[ridx].cpu().numpy().astype(np.float64)
    Wt, Wi = wl.w_train.cpu(), wl.w_infer.cpu()
    ot = orc.lmhead(H, Wt, ids, np.float32(lr), grad_out=g, band=BAND, want_flags=True, threads=8)
    oi = orc.lmhead(H, Wi, ids, np.float32(lr), band=BAND, threads=8)

    class Sub:
        pass

    def cut(side):
        s = Sub()
        for k in ("logp", "row_max", "lse_safe", "safe_count"):
            setattr(s, k, getattr(side, k)[ridx])
        s.lse_full = None
        return s

    _check_side("train", cut(res.train), ot, ot)
    _check_side("infer", cut(res.infer), oi, oi)
    clean = (ot["band_count"] == 0) & (ot["y_in_safe"] == 1) & (ot["safe_count"] <= cap)
    assert clean.sum() >= 30
    W64 = Wt.double().numpy()
    dz_round = 2.0 ** -19 * (np.abs(ot["row_max"]).max() + 10.0)
    dh = res.d_hidden[ridx].cpu().double().numpy()
    for j in np.nonzero(clean)[0]:
        idx, val = res.row(int(rows[j]))
        want = np.nonzero(ot["safe_flags"][j])[0]
        np.testing.assert_array_equal(idx.numpy(), want)
        ref = ot["dz"][j, want]
        pk = np.abs(ref).copy()
        pk[want == ids[j]] = abs(g[j]) * np.exp(ot["logp"][j])
        assert np.all(np.abs(val.double().numpy() - ref) <= 2 * dz_round * pk + 1e-6 * max(1.0, abs(g[j])))
        bound = 2 * dz_round * (pk @ np.abs(W64[want])) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_hidden"][j])
        assert (np.abs(dh[j] - ot["d_hidden"][j]) / bound).max() <= 1.0
        assert np.abs(dh[j] - ot["d_hidden"][j]).max() <= 2e-3
    # any-size properties on every row and token
    flags = res.row_flags
    over = (flags & dvp.ROW_GRAD_OVERFLOW) != 0
    glen = torch.where(over, torch.zeros_like(res.grad_len), res.grad_len)
    assert torch.all(res.train.safe_count >= 1)
    assert torch.equal(res.grad_len, torch.where((flags & 1) != 0, res.train.safe_count, torch.zeros_like(res.grad_len)))
    assert torch.isfinite(res.d_w).all() and torch.isfinite(res.d_hidden).all()
    valid = torch.arange(cap, device="cuda")[None, :] < glen[:, None]
    tok = (res.entries[..., 0].to(torch.int64) & 0xFFFFFFFF)[valid]
    val = res.entries[..., 1].contiguous().view(torch.float32)[valid].double()
    row_of = torch.arange(n, device="cuda")[:, None].expand(n, cap)[valid]
    touched = torch.zeros(v, dtype=torch.bool, device="cuda")
    touched[tok] = True
    assert torch.all(res.d_w[~touched] == 0.0)
    used = torch.nonzero(touched).squeeze(1)
    slot = torch.full((v,), -1, dtype=torch.int64, device="cuda")
    slot[used] = torch.arange(used.numel(), device="cuda")
    want_w = torch.zeros(used.numel(), d, dtype=torch.float64, device="cuda")
    for s0 in range(0, tok.numel(), 8192):                 # in pieces: the products are [pieces, d] fp64
        sl = slice(s0, s0 + 8192)
        want_w.index_add_(0, slot[tok[sl]], val[sl, None] * wl.hidden[row_of[sl]].double())
    got_w = res.d_w[used].double()
    assert (got_w - want_w).abs().max().item() <= 1e-5 + 2.0 ** -18 * want_w.abs().max().item()
    col = res.d_w.double().sum(dim=0).abs().max().item()
    scale = res.d_w.double().abs().sum(dim=0).max().item()
    assert col <= 2.0 ** -16 * scale
    del wl, res
    torch.cuda.empty_cache()
