"""Element-by-element comparison of the HIP row path with the fp64 oracle.

Tolerances (absolute): log-probs, lse: 1e-5 for fp32 inputs, 2e-3 for bf16
inputs.  Gradients: fp32 output 1e-5 * max(1, |grad_out_i|); bf16 output
max(2e-3, half_ulp_bf16(|dz_oracle|) + 1e-5 * max(1, |grad_out_i|)) -- the
gradient is stored with 8 significant bits, so an element of magnitude >= 1
cannot be closer than 2^-8 to the exact value whatever the kernel computes;
below magnitude 1 the bound is the plain 2e-3.  Row maxima, safe-set sizes and
membership must match exactly: both sides decide membership by the same fp32
threshold fl32(m + log_rho).
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import dvp_oracle as orc

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3}


def to_host(t):
    return None if t is None else t.detach().cpu()


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def check_side(name, gpu_side, z_host, ids_host, log_rho, tol, vocab, rows=None,
               check_bits=True, threads=8):
    """Compare one side's per-row outputs on `rows` (default: all) against the oracle.
    Returns a dict of statistics; raises AssertionError on any mismatch."""
    n = z_host.shape[0]
    sel = np.arange(n) if rows is None else np.asarray(rows)
    zs = z_host[torch.as_tensor(sel)]
    ids_s = ids_host.numpy()[sel]
    want_bits = check_bits and gpu_side.safe_bits is not None
    o = orc.rows(zs, ids_s, np.float32(log_rho), want_flags=want_bits, threads=threads)

    got_max = f64(gpu_side.row_max)[sel]
    np.testing.assert_array_equal(got_max, o["row_max"], err_msg=name + ": row_max")
    got_cnt = gpu_side.safe_count.cpu().numpy()[sel]
    np.testing.assert_array_equal(got_cnt, o["safe_count"], err_msg=name + ": safe_count")

    got_lse = f64(gpu_side.lse_safe)[sel]
    err_lse = np.abs(got_lse - o["lse_safe"]).max()
    assert err_lse <= tol, "%s: lse_safe max abs err %.3e > %.1e" % (name, err_lse, tol)
    err_full = 0.0
    if gpu_side.lse_full is not None:
        err_full = np.abs(f64(gpu_side.lse_full)[sel] - o["lse_full"]).max()
        assert err_full <= tol, "%s: lse_full max abs err %.3e > %.1e" % (name, err_full, tol)

    got_lp = f64(gpu_side.logp)[sel]
    want_lp = o["logp"]
    fin = np.isfinite(want_lp)
    np.testing.assert_array_equal(np.isneginf(got_lp), np.isneginf(want_lp), err_msg=name + ": -inf logp")
    np.testing.assert_array_equal(np.isnan(got_lp), np.isnan(want_lp), err_msg=name + ": NaN logp")
    err_lp = np.abs(got_lp[fin] - want_lp[fin]).max() if fin.any() else 0.0
    assert err_lp <= tol, "%s: logp max abs err %.3e > %.1e" % (name, err_lp, tol)

    if want_bits:
        got_flags = gpu_side.flags_matrix(vocab).cpu().numpy()[sel]
        np.testing.assert_array_equal(got_flags, o["safe_flags"], err_msg=name + ": membership")
        words = gpu_side.safe_bits.cpu().numpy().view(np.uint32)[sel]
        used = vocab % 32
        if used:
            assert np.all((words[:, -1] >> used) == 0), name + ": stray bits past V"
    return dict(err_lse=float(err_lse), err_full=float(err_full), err_logp=float(err_lp),
                band_tokens=int(o["band_count"].sum()), y_in_safe=o["y_in_safe"],
                safe_count=o["safe_count"])


def check_flags(row_flags, y_train_safe, y_infer_safe, ids_host, vocab, rows=None, train_safe_count=None):
    """train_safe_count: the oracle's safe-set sizes of the training side; given, the short-safe-set bit
    (at most 64 tokens) is checked as well, else it is ignored."""
    got = row_flags.cpu().numpy()
    if train_safe_count is None:
        got = got & ~np.uint8(16)
    if rows is not None:
        got = got[np.asarray(rows)]
        ids = ids_host.numpy()[np.asarray(rows)]
    else:
        ids = ids_host.numpy()
    want = y_train_safe.astype(np.uint8) * 1
    if y_infer_safe is not None:
        want = want | (y_infer_safe.astype(np.uint8) * 2)
    want = want | (((ids < 0) | (ids >= vocab)).astype(np.uint8) * 4)
    if train_safe_count is not None:
        want = want | ((np.asarray(train_safe_count) <= 64).astype(np.uint8) * 16)
    np.testing.assert_array_equal(got, want, err_msg="row_flags")


def check_gradient(name, dz_gpu, z_host, ids_host, grad_host, log_rho, tol, rows=None, threads=8):
    n = z_host.shape[0]
    sel = np.arange(n) if rows is None else np.asarray(rows)
    zs = z_host[torch.as_tensor(sel)]
    g = grad_host.numpy().astype(np.float64)[sel]
    o = orc.rows(zs, ids_host.numpy()[sel], np.float32(log_rho), grad_out=g, want_dz=True,
                 want_flags=True, threads=threads)
    got = f64(dz_gpu[torch.as_tensor(sel).to(dz_gpu.device)])
    scale = np.maximum(1.0, np.abs(g))[:, None]
    if dz_gpu.dtype == torch.bfloat16:
        mag = np.abs(o["dz"])
        with np.errstate(divide="ignore"):
            half_ulp = np.where(mag > 0, np.exp2(np.floor(np.log2(np.maximum(mag, 1e-300))) - 8), 0.0)
        bound = np.maximum(tol, half_ulp + 1e-5 * scale)
    else:
        bound = tol * scale
    err = np.abs(got - o["dz"]) / bound
    worst = err.max() if err.size else 0.0
    assert worst <= 1.0, "%s: gradient error is %.3f x its bound (raw max abs %.3e)" % (
        name, worst, np.abs(got - o["dz"]).max())
    # exact zeros off the safe set and on rows whose sampled token is pruned
    off = o["safe_flags"] == 0
    assert np.all(got[off] == 0.0), name + ": nonzero gradient outside the safe set"
    assert np.all(got[o["y_in_safe"] == 0] == 0.0), name + ": nonzero gradient on a pruned-token row"
    return dict(err_grad=float(worst), raw_err=float(np.abs(got - o["dz"]).max() if err.size else 0.0))


# ---------------------------------------------------------------------------
# Bulk comparison for whole workloads (bench.py's parity leg, the full-size tests): walks the rows in
# chunks, counts instead of raising, and keeps the time spent inside the oracle so that the same pass
# serves as the CPU baseline.  torch CPU ops do the element-wise comparisons (they use every host core).
# ---------------------------------------------------------------------------
import time


class RowParity:
    """Accumulates the comparison of one dvp_forward_backward call's outputs with the oracle."""

    def __init__(self, log_rho, dtype, vocab, threads=8):
        self.log_rho, self.dtype, self.vocab, self.threads = np.float32(log_rho), dtype, vocab, threads
        self.tol = TOL[dtype]
        self.rows = 0
        self.oracle_seconds = 0.0
        self.c = dict(row_max_mismatches=0, safe_count_mismatches=0, membership_bit_mismatches=0,
                      membership_rows_checked=0, row_flag_mismatches=0, logp_inf_nan_mismatches=0,
                      grad_nonzero_outside_safe_set=0, grad_nonzero_on_pruned_token_rows=0,
                      rows_sampled_token_pruned_train=0, rows_sampled_token_pruned_infer=0,
                      band_tokens_train=0, band_tokens_infer=0)
        self.m = dict(logp_max_abs_err=0.0, lse_safe_max_abs_err=0.0, lse_full_max_abs_err=0.0,
                      grad_worst_ratio_to_bound=0.0, grad_raw_max_abs_err=0.0)

    def _side(self, name, got, o):
        """got: dict of host numpy arrays for one side (row_max, safe_count, lse_safe, logp[, lse_full])."""
        self.c["row_max_mismatches"] += int((got["row_max"].astype(np.float64) != o["row_max"]).sum())
        self.c["safe_count_mismatches"] += int((got["safe_count"] != o["safe_count"]).sum())
        self.m["lse_safe_max_abs_err"] = max(self.m["lse_safe_max_abs_err"],
                                             float(np.abs(got["lse_safe"].astype(np.float64) - o["lse_safe"]).max()))
        if got.get("lse_full") is not None:
            self.m["lse_full_max_abs_err"] = max(self.m["lse_full_max_abs_err"],
                                                 float(np.abs(got["lse_full"].astype(np.float64) - o["lse_full"]).max()))
        lp, want = got["logp"].astype(np.float64), o["logp"]
        self.c["logp_inf_nan_mismatches"] += int((np.isneginf(lp) != np.isneginf(want)).sum()
                                                 + (np.isnan(lp) != np.isnan(want)).sum())
        fin = np.isfinite(want) & np.isfinite(lp)
        if fin.any():
            self.m["logp_max_abs_err"] = max(self.m["logp_max_abs_err"], float(np.abs(lp[fin] - want[fin]).max()))
        self.c["band_tokens_" + name] += int(o["band_count"].sum())
        self.c["rows_sampled_token_pruned_" + name] += int((o["y_in_safe"] == 0).sum())

    def add_chunk(self, z_train, z_infer, ids, grad_out, train, infer, row_flags, dz, bits_train=None,
                  bits_infer=None):
        """One chunk of rows, everything on the host: z_* CPU tensors [m, V]; ids int64 numpy [m];
        grad_out float numpy [m]; train / infer dicts of numpy arrays; row_flags uint8 numpy [m];
        dz CPU tensor [m, V] or None; bits_* uint32 numpy [m, ceil(V/32)] or None."""
        m, v = z_train.shape
        g = None if grad_out is None else grad_out.astype(np.float64)
        want_dz = dz is not None
        t0 = time.perf_counter()
        ot = orc.rows(z_train, ids, self.log_rho, grad_out=g if want_dz else None, want_dz=want_dz,
                      want_flags=want_dz or bits_train is not None, threads=self.threads)
        oi = orc.rows(z_infer, ids, self.log_rho, want_flags=bits_infer is not None, threads=self.threads)
        self.oracle_seconds += time.perf_counter() - t0
        self.rows += m
        self._side("train", train, ot)
        self._side("infer", infer, oi)
        want_flags = (ot["y_in_safe"].astype(np.uint8) | (oi["y_in_safe"].astype(np.uint8) << 1)
                      | (((ids < 0) | (ids >= v)).astype(np.uint8) << 2)
                      | ((ot["safe_count"] <= 64).astype(np.uint8) << 4))      # the short-safe-set bit
        self.c["row_flag_mismatches"] += int((row_flags != want_flags).sum())
        for bits, o in ((bits_train, ot), (bits_infer, oi)):
            if bits is not None:
                got = np.unpackbits(bits.view(np.uint8), axis=1, bitorder="little")[:, :v]
                self.c["membership_bit_mismatches"] += int((got != o["safe_flags"]).sum())
                self.c["membership_rows_checked"] += m
        if want_dz:
            want = torch.from_numpy(ot["dz"])
            flags = torch.from_numpy(ot["safe_flags"])
            nz_got = dz != 0
            self.c["grad_nonzero_outside_safe_set"] += int((nz_got & (flags == 0)).sum().item())
            pruned = torch.from_numpy(ot["y_in_safe"] == 0)
            if pruned.any():
                self.c["grad_nonzero_on_pruned_token_rows"] += int(nz_got[pruned].sum().item())
            either = nz_got | (want != 0)
            if int(either.sum().item()) * 5 > either.numel():      # dense rows: compare whole matrices
                gv, wv = dz.to(torch.float64).reshape(-1), want.reshape(-1)
                scale = torch.from_numpy(np.maximum(1.0, np.abs(g)))[:, None].expand(m, v).reshape(-1)
            else:                                                   # short safe sets: only the entries that exist
                r, c = torch.nonzero(either, as_tuple=True)
                gv, wv = dz[r, c].to(torch.float64), want[r, c]
                scale = torch.from_numpy(np.maximum(1.0, np.abs(g)))[r]
            if gv.numel():
                if self.dtype == torch.bfloat16:     # half a unit in the last place of a bf16 of wv's magnitude
                    expo = torch.frexp(wv.abs()).exponent.to(torch.float64)
                    half_ulp = torch.where(wv != 0, torch.exp2(expo - 1.0 - 8.0), torch.zeros_like(wv))
                    bound = torch.clamp(half_ulp + 1e-5 * scale, min=self.tol)
                else:
                    bound = self.tol * scale
                err = (gv - wv).abs()
                self.m["grad_worst_ratio_to_bound"] = max(self.m["grad_worst_ratio_to_bound"], float((err / bound).max()))
                self.m["grad_raw_max_abs_err"] = max(self.m["grad_raw_max_abs_err"], float(err.max()))

    def result(self):
        out = dict(rows_checked=self.rows, **self.c, **self.m)
        out["tolerance"] = {"logp_lse_abs": self.tol,
                            "grad": "fp32: 1e-5 max(1,|g|); bf16: max(2e-3, half ulp of the bf16 nearest the exact value "
                                    "+ 1e-5 max(1,|g|)); integers, row maxima, membership and flags exact"}
        exact = ("row_max_mismatches", "safe_count_mismatches", "membership_bit_mismatches", "row_flag_mismatches",
                 "logp_inf_nan_mismatches", "grad_nonzero_outside_safe_set", "grad_nonzero_on_pruned_token_rows")
        out["ok"] = bool(all(self.c[k] == 0 for k in exact) and self.m["logp_max_abs_err"] <= self.tol
                         and self.m["lse_safe_max_abs_err"] <= self.tol and self.m["lse_full_max_abs_err"] <= self.tol
                         and self.m["grad_worst_ratio_to_bound"] <= 1.0)
        return out


def side_arrays(side, sel):
    """Host numpy arrays of one side's outputs on the rows `sel` (a slice or an index tensor on the device)."""
    out = {}
    for k in ("row_max", "safe_count", "lse_safe", "logp", "lse_full"):
        t = getattr(side, k)
        out[k] = None if t is None else t[sel].cpu().numpy()
    return out


def compare_workload(wl, log_rho, train, infer, row_flags, dz, rows=None, chunk=512, threads=8, bits=None):
    """Walk `rows` (an increasing int64 numpy array; default every row) of a row workload in chunks and
    compare the given call's outputs with the oracle.  bits = (train SideOutputs, infer SideOutputs) of a
    call with safe_bits, or None.  Returns the RowParity (result(), oracle_seconds)."""
    n, v = wl.z_train.shape
    rp = RowParity(log_rho, wl.z_train.dtype, v, threads=threads)
    all_rows = rows is None
    total = n if all_rows else len(rows)
    dev = wl.z_train.device
    for c0 in range(0, total, chunk):
        c1 = min(total, c0 + chunk)
        sel = slice(c0, c1) if all_rows else torch.as_tensor(rows[c0:c1], device=dev)
        g = None if wl.grad_out is None else wl.grad_out[sel].cpu().numpy()
        rp.add_chunk(wl.z_train[sel].cpu(), wl.z_infer[sel].cpu(), wl.ids[sel].cpu().numpy(), g,
                     side_arrays(train, sel), side_arrays(infer, sel), row_flags[sel].cpu().numpy(),
                     None if dz is None else dz[sel].cpu(),
                     None if bits is None else bits[0].safe_bits[sel].cpu().numpy().view(np.uint32),
                     None if bits is None else bits[1].safe_bits[sel].cpu().numpy().view(np.uint32))
    return rp


# ---------------------------------------------------------------------------
# LM-head variant on sampled token rows of a large workload: forward outputs of both sides and the rows
# of dH against the oracle (fp64 logits from the stored H and W: V * d multiply-adds per row and side).
# The matrix cores accumulate each logit in fp32, so it differs from the oracle's by accumulation
# rounding; membership can only be compared outside a band around the threshold (`band`, in logit
# units; the oracle counts the tokens inside it per row).
# ---------------------------------------------------------------------------
def lmhead_sampled_rows(wl, res, rows, log_rho, band=2e-4, threads=8, infer_scale=None):
    """Returns (dict of error figures with 'ok', seconds spent inside the oracle).  `res` is the result of
    the GPU call on the whole workload (d_hidden may be None for a forward-only call); `infer_scale`
    not None: the inference side is the 8-bit engine (wl.hidden8, wl.w8) with that dequantisation factor."""
    idx = torch.as_tensor(rows, device=wl.hidden.device)
    H = wl.hidden[idx].cpu()
    ids = wl.ids[idx].cpu().numpy()
    g = wl.grad_out[idx].cpu().numpy().astype(np.float64)
    grad = res.d_hidden is not None
    Wt = wl.w_train.cpu()
    t0 = time.perf_counter()
    ot = orc.lmhead(H, Wt, ids, np.float32(log_rho), grad_out=g if grad else None, band=band, threads=threads)
    if infer_scale is None:
        oi = orc.lmhead(H, wl.w_infer.cpu(), ids, np.float32(log_rho), band=band, threads=threads)
    else:
        oi = orc.lmhead(wl.hidden8[idx].cpu(), wl.w8.cpu(), ids, np.float32(log_rho), band=band, threads=threads,
                        scale=infer_scale)
    seconds = time.perf_counter() - t0
    out = dict(rows_checked=len(rows), band_logit_units=band, band_tokens_train=int(ot["band_count"].sum()),
               band_tokens_infer=int(oi["band_count"].sum()))
    ok = True
    for name, side, o in (("train", res.train, ot), ("infer", res.infer, oi)):
        m = side.row_max[idx].cpu().double().numpy()
        out[name + "_row_max_max_abs_err"] = float(np.abs(m - o["row_max"]).max())
        cnt = side.safe_count[idx].cpu().numpy()
        over = np.abs(cnt - o["safe_count"]) > o["band_count"]
        out[name + "_safe_count_beyond_band_rows"] = int(over.sum())
        lse = side.lse_safe[idx].cpu().double().numpy()
        out[name + "_lse_safe_max_abs_err"] = float(np.abs(lse - o["lse_safe"]).max())
        lp = side.logp[idx].cpu().double().numpy()
        same = np.isfinite(lp) == np.isfinite(o["logp"])
        out[name + "_logp_side_flips_outside_band"] = int(max(0, (~same).sum() - (o["band_count"] > 0).sum()))
        fin = same & np.isfinite(o["logp"])
        out[name + "_logp_max_abs_err"] = float(np.abs(lp[fin] - o["logp"][fin]).max()) if fin.any() else 0.0
        ok = ok and out[name + "_row_max_max_abs_err"] <= band and not over.any() and \
            out[name + "_lse_safe_max_abs_err"] <= 2e-3 and out[name + "_logp_max_abs_err"] <= 2e-3 and \
            out[name + "_logp_side_flips_outside_band"] == 0
        if name == "train":
            same_t = same
    if grad:
        W64 = Wt.double().numpy()
        soft = np.abs(ot["dz"])                        # |c| p of every token but the sampled one: the part that passes through bf16
        safe_rows = np.nonzero(ot["y_in_safe"])[0]
        soft[safe_rows, ids[safe_rows]] = 0.0
        bound_h = 2.0 ** -8 * (soft @ np.abs(W64)) + 1e-5 + 2.0 ** -20 * np.abs(ot["d_hidden"])
        dh = res.d_hidden[idx].cpu().double().numpy()
        err = np.abs(dh - ot["d_hidden"])[same_t]
        out["d_hidden_worst_ratio_to_bound"] = float((err / bound_h[same_t]).max())
        out["d_hidden_max_abs_err"] = float(err.max())
        ok = ok and out["d_hidden_worst_ratio_to_bound"] <= 1.0 and out["d_hidden_max_abs_err"] <= 2e-3
    out["ok"] = bool(ok)
    return out, seconds
