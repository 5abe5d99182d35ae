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


def check_flags(row_flags, y_train_safe, y_infer_safe, ids_host, vocab, rows=None):
    got = row_flags.cpu().numpy()
    if rows is not None:
        got = got[np.asarray(rows)]
        ids = ids_host.numpy()[np.asarray(rows)]
    else:
        ids = ids_host.numpy()
    want = y_train_safe.astype(np.uint8) * 1
    if y_infer_safe is not None:
        want = want | (y_infer_safe.astype(np.uint8) * 2)
    want = want | (((ids < 0) | (ids >= vocab)).astype(np.uint8) * 4)
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
