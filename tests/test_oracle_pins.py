"""Pins for the fp64 CPU oracle: each test checks it against something the
paper or the mathematics fixes, computed here without the oracle's code
(scipy / torch library routines, probability-space brute force, autograd,
finite differences, closed-form identities)."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import dvp_oracle as orc
from paper_2512_23087_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_rows(n, v, seed, scale=3.0, dtype=np.float64):
    rng = np.random.default_rng(seed)
    z = (scale * rng.standard_normal((n, v))).astype(dtype)
    ids = rng.integers(0, v, size=n)
    return z, ids


# --------------------------------------------------------------------------
# printed constants (Sec. 5.1, Sec. 5.5, App. A)
# --------------------------------------------------------------------------
def test_printed_constants():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val, tol = line.split()
            vals[name] = (float(val), float(tol))
    for name in ("exp_minus_13_sec5_1", "exp_minus_13_sec5_5"):
        v, tol = vals[name]
        assert abs(math.exp(-13.0) - v) <= tol * v
        assert abs(float(np.exp(np.float64(orc.log_rho_f32(math.exp(-13.0))))) - v) <= tol * v
    v, tol = vals["exp_minus_50_appA"]
    assert abs(math.exp(-50.0) - v) <= tol * v
    # log_rho helper: single fp32 constant, rho = 0 means no pruning
    assert orc.log_rho_f32(math.exp(-13.0)) == np.float32(-13.0)
    assert orc.log_rho_f32(1.0) == np.float32(0.0)
    assert orc.log_rho_f32(0.0) == np.float32(-np.inf)
    with pytest.raises(ValueError):
        orc.log_rho_f32(1.5)


# --------------------------------------------------------------------------
# empty prune set reproduces the full log-softmax exactly (Prop. 5.6 with V_S = V)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_no_pruning_is_full_log_softmax(dtype):
    z, ids = _rand_rows(17, 1000, 1, dtype=dtype)
    out = orc.rows(z, ids, orc.log_rho_f32(0.0), want_flags=True)
    z64 = z.astype(np.float64)
    lse = scipy.special.logsumexp(z64, axis=1)
    lsm = torch.log_softmax(torch.from_numpy(z64), dim=-1).numpy()
    assert np.all(out["safe_count"] == z.shape[1])
    assert np.all(out["safe_flags"] == 1)
    assert np.all(out["y_in_safe"] == 1)
    np.testing.assert_allclose(out["lse_safe"], lse, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["lse_full"], lse, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["logp"], lsm[np.arange(len(ids)), ids], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(out["row_max"], z64.max(axis=1))


# --------------------------------------------------------------------------
# masked case against library routines on an independently built mask
# --------------------------------------------------------------------------
@pytest.mark.parametrize("rho", [1e-1, 1e-2, 1e-4, math.exp(-13.0), 1.0])
def test_masked_lse_against_scipy_and_torch(rho):
    z, ids = _rand_rows(33, 777, 2, dtype=np.float32)
    lr = orc.log_rho_f32(rho)
    out = orc.rows(z, ids, lr, want_flags=True)
    # threshold: one fp32 add of the row max and the fp32 constant (App. A item 2)
    thr = (z.max(axis=1) + lr).astype(np.float32)
    mask = z >= thr[:, None]
    z64 = z.astype(np.float64)
    np.testing.assert_array_equal(out["safe_flags"].astype(bool), mask)
    np.testing.assert_array_equal(out["safe_count"], mask.sum(axis=1))
    np.testing.assert_array_equal(out["tau"], thr.astype(np.float64))
    lse_m = scipy.special.logsumexp(z64, axis=1, b=mask.astype(np.float64))
    np.testing.assert_allclose(out["lse_safe"], lse_m, rtol=0, atol=1e-12)
    # Prop. 5.6 part 1: the constrained policy is the softmax of the logits with -inf outside the safe set
    outside = np.full_like(z64, -np.inf)
    outside[mask] = z64[mask]
    lsm = scipy.special.log_softmax(outside, axis=1)
    want = lsm[np.arange(len(ids)), ids]
    np.testing.assert_allclose(out["logp"], want, rtol=0, atol=1e-12)  # -inf == -inf passes
    np.testing.assert_array_equal(out["y_in_safe"].astype(bool), mask[np.arange(len(ids)), ids])
    # coverage mass log Z = lse_safe - lse_full <= 0
    p = scipy.special.softmax(z64, axis=1)
    np.testing.assert_allclose(np.exp(out["lse_safe"] - out["lse_full"]),
                               (p * mask).sum(axis=1), rtol=1e-12)


# --------------------------------------------------------------------------
# brute force in probability space on tiny vocabularies (Def. 5.1 / 5.2 as written)
# --------------------------------------------------------------------------
def test_bruteforce_probability_space_tiny_vocab():
    rng = np.random.default_rng(3)
    checked = 0
    for trial in range(400):
        v = int(rng.integers(1, 17))
        z = (4.0 * rng.standard_normal(v)).astype(np.float32)
        rho = float(10.0 ** rng.uniform(-6, 0))
        y = int(rng.integers(0, v))
        z64 = z.astype(np.float64)
        pi = np.exp(z64 - z64.max())
        pi /= pi.sum()
        ratio = pi / (rho * pi.max())
        if np.any(np.abs(ratio - 1.0) < 1e-5):
            continue  # on the boundary: the two spaces may round differently
        safe = pi >= rho * pi.max()
        pmp = np.where(safe, pi, 0.0) / pi[safe].sum()
        out = orc.rows(z[None, :], [y], orc.log_rho_f32(rho), want_flags=True, want_dz=True,
                       grad_out=[1.0])
        np.testing.assert_array_equal(out["safe_flags"][0].astype(bool), safe)
        assert out["safe_count"][0] == safe.sum()
        if safe[y]:
            assert abs(out["logp"][0] - math.log(pmp[y])) < 1e-12
            onehot = np.zeros(v)
            onehot[y] = 1.0
            np.testing.assert_allclose(out["dz"][0], onehot - pmp, rtol=0, atol=1e-12)
        else:
            assert out["logp"][0] == -np.inf
            assert np.all(out["dz"][0] == 0.0)
        assert abs(math.exp(out["lse_safe"][0] - out["lse_full"][0]) - pi[safe].sum()) < 1e-12
        checked += 1
    assert checked > 300


# --------------------------------------------------------------------------
# invariants from the definitions
# --------------------------------------------------------------------------
def test_invariants_and_nestedness():
    wl = workloads.make_rows(0, n=16, v=4000)
    z = wl.z_train.numpy()
    ids = wl.ids.numpy()
    prev_flags = None
    for rho in [0.0, 1e-6, 1e-4, 1e-2, 1.0]:
        out = orc.rows(z, ids, orc.log_rho_f32(rho), want_flags=True, want_dz=True,
                       grad_out=np.ones(len(ids)))
        f = out["safe_flags"].astype(bool)
        c = out["safe_count"]
        assert np.all(c >= 1) and np.all(c <= z.shape[1])
        assert np.all(f[np.arange(len(ids)), z.argmax(axis=1)])          # arg max is always safe
        assert np.all(out["row_max"] <= out["lse_safe"] + 1e-15)
        assert np.all(out["lse_safe"] <= out["row_max"] + np.log(c) + 1e-12)
        assert np.all(out["lse_safe"] <= out["lse_full"] + 1e-15)
        # constrained probabilities sum to one and vanish off the safe set (Def. 5.2)
        pmp = np.where(f, np.exp(z.astype(np.float64) - out["lse_safe"][:, None]), 0.0)
        np.testing.assert_allclose(pmp.sum(axis=1), 1.0, rtol=0, atol=1e-12)
        # pruned mass floor: every pruned token has pi < rho * pi_max
        pmax = np.exp(out["row_max"] - out["lse_full"])
        one_minus_z = -np.expm1(out["lse_safe"] - out["lse_full"])
        assert np.all(one_minus_z <= (z.shape[1] - c) * rho * pmax + 1e-15)
        # gradient: sums to zero, zero off the set, zero row when y is pruned (Prop. 5.4)
        ys = out["y_in_safe"].astype(bool)
        np.testing.assert_allclose(out["dz"][ys].sum(axis=1), 0.0, atol=1e-12)
        assert np.all(out["dz"][~f] == 0.0)
        assert np.all(out["dz"][~ys] == 0.0)
        if rho == 1.0:
            assert np.all(f == (z == z.max(axis=1, keepdims=True)))
        if prev_flags is not None:
            assert np.all(prev_flags | ~f)     # larger rho => subset
        prev_flags = f


def test_threshold_boundary_is_inclusive_and_ties():
    # element exactly at the threshold is safe (Def. 5.1 uses >=); ties at the max are all safe
    lr = np.float32(-2.0)
    z = np.array([[4.0, 2.0, 1.9999999, 4.0, -np.inf, 2.0000002]], dtype=np.float32)
    out = orc.rows(z, [1], lr, want_flags=True)
    np.testing.assert_array_equal(out["safe_flags"][0], [1, 1, 0, 1, 0, 1])
    assert out["safe_count"][0] == 4 and out["y_in_safe"][0] == 1
    want = 2.0 - math.log(2 * math.exp(4.0) + math.exp(2.0) + math.exp(float(np.float32(2.0000002))))
    assert abs(out["logp"][0] - want) < 1e-12
    # all-equal row: everything is safe at any rho
    z = np.full((1, 37), -3.25, dtype=np.float32)
    out = orc.rows(z, [5], orc.log_rho_f32(1.0))
    assert out["safe_count"][0] == 37
    assert abs(out["logp"][0] + math.log(37)) < 1e-12
    # single element vocabulary
    out = orc.rows(np.array([[0.7]], dtype=np.float32), [0], orc.log_rho_f32(1e-3))
    assert out["safe_count"][0] == 1 and out["logp"][0] == 0.0
    # out-of-range id: NaN log-prob, not in the set
    out = orc.rows(z, [37], orc.log_rho_f32(1e-3), want_dz=True)
    assert np.isnan(out["logp"][0]) and out["y_in_safe"][0] == 0 and np.all(out["dz"] == 0)


def test_band_count():
    lr = np.float32(-1.0)
    z = np.array([[3.0, 2.0, 2.0000005, 1.9999995, 2.00001, 0.0]], dtype=np.float64)
    out = orc.rows(z, [0], lr, band=1e-6)
    assert out["band_count"][0] == 3


def test_bf16_inputs_are_widened_exactly():
    t = (3.0 * torch.randn(5, 300, generator=torch.Generator().manual_seed(4))).to(torch.bfloat16)
    ids = np.arange(5)
    a = orc.rows(t, ids, orc.log_rho_f32(1e-2), want_flags=True, want_dz=True)
    b = orc.rows(t.to(torch.float64).numpy(), ids, orc.log_rho_f32(1e-2), want_flags=True,
                 want_dz=True)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_e4m3_codes_against_the_format_definition_and_torch():
    """The 8-bit E4M3 decode (inference logits of an FP8 engine, Sec. 4.2) against facts the OCP
    format fixes and against torch's own float8_e4m3fn widening of all 256 codes."""
    val = np.array([orc.e4m3_value(c) for c in range(256)])
    # facts of the format: 1.0, the largest finite value 448, the smallest normal 2^-6, the
    # smallest subnormal 2^-9, one NaN per sign and no infinity, two zeros
    assert val[0x38] == 1.0 and val[0x7E] == 448.0 and val[0x08] == 2.0 ** -6 and val[0x01] == 2.0 ** -9
    assert val[0x00] == 0.0 and val[0x80] == 0.0 and np.signbit(val[0x80])
    assert np.isnan(val[0x7F]) and np.isnan(val[0xFF]) and np.isnan(val).sum() == 2
    assert not np.isinf(val).any()
    pos = val[:0x7F]
    assert np.all(np.diff(pos) > 0)                       # codes order like their values
    np.testing.assert_array_equal(val[0x80:0xFF], -pos)   # the sign bit only flips the sign
    # subnormals are evenly spaced, and each binade holds 8 evenly spaced values
    np.testing.assert_array_equal(val[0:8], np.arange(8) * 2.0 ** -9)
    for e in range(1, 16):
        top = 8 if e < 15 else 7
        np.testing.assert_array_equal(val[8 * e:8 * e + top], 2.0 ** (e - 7) * (1 + np.arange(top) / 8))
    # torch's conversion of the same bit patterns
    t = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(np.isnan(t), np.isnan(val))
    ok = ~np.isnan(val)
    np.testing.assert_array_equal(t[ok], val[ok])
    assert np.array_equal(np.signbit(t[ok]), np.signbit(val[ok]))


def test_e4m3_inputs_are_widened_exactly():
    g = torch.Generator().manual_seed(9)
    t = (3.0 * torch.randn(6, 333, generator=g)).to(torch.float8_e4m3fn)
    ids = np.arange(6)
    a = orc.rows(t, ids, orc.log_rho_f32(1e-2), want_flags=True)
    b = orc.rows(t.to(torch.float64).numpy(), ids, orc.log_rho_f32(1e-2), want_flags=True)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    # and as raw codes in a numpy array
    c = orc.rows(t.view(torch.uint8).numpy(), ids, orc.log_rho_f32(1e-2), want_flags=True)
    for k in a:
        np.testing.assert_array_equal(a[k], c[k])


def test_lmhead_oracle_with_an_8bit_inference_engine():
    """Logits of an 8-bit engine, scale * hidden8 w8^T on E4M3 codes, equal the logits of the dequantised
    matrices (s_h hidden8)(s_w w8)^T; torch's own float8 widening supplies the dequantised values."""
    g = torch.Generator().manual_seed(21)
    h = torch.randn(7, 64, generator=g)
    w = 0.02 * torch.randn(50, 64, generator=g)
    s_h, s_w = float(h.abs().max()) / 448.0, float(w.abs().max()) / 448.0
    h8 = (h / s_h).to(torch.float8_e4m3fn)
    w8 = (w / s_w).to(torch.float8_e4m3fn)
    ids = np.arange(7)
    lr = orc.log_rho_f32(1e-3)
    a = orc.lmhead(h8, w8, ids, lr, scale=s_h * s_w)
    b = orc.lmhead((h8.to(torch.float64) * s_h).numpy(), (w8.to(torch.float64) * s_w).numpy(), ids, lr)
    np.testing.assert_allclose(a["z"], b["z"], rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(a["safe_count"], b["safe_count"])
    np.testing.assert_allclose(a["logp"], b["logp"], rtol=0, atol=1e-12)
    assert np.abs(a["z"]).max() > 0.1        # not a comparison of zeros
    with pytest.raises(ValueError):
        orc.lmhead(h8, w8, ids, lr, grad_out=np.ones(7), scale=2.0)


def test_shift_invariance():
    z, ids = _rand_rows(8, 500, 5)
    lr = orc.log_rho_f32(1e-3)
    a = orc.rows(z, ids, lr, want_flags=True, want_dz=True)
    # shift by a power of two keeps the fp32 threshold rounding aligned for these magnitudes
    zf = z.astype(np.float32).astype(np.float64)
    a = orc.rows(zf, ids, lr, want_flags=True, want_dz=True)
    b = orc.rows(zf + 64.0, ids, lr, want_flags=True, want_dz=True)
    agree = np.abs(zf - a["tau"][:, None]).min(axis=1) > 1e-4   # rows with nothing near the threshold
    assert agree.sum() >= 6
    np.testing.assert_array_equal(a["safe_flags"][agree], b["safe_flags"][agree])
    np.testing.assert_allclose(a["logp"][agree], b["logp"][agree], atol=1e-12)
    np.testing.assert_allclose(a["lse_safe"][agree] + 64.0, b["lse_safe"][agree], atol=1e-11)
    np.testing.assert_allclose(a["dz"][agree], b["dz"][agree], atol=1e-12)


# --------------------------------------------------------------------------
# gradient: autograd through the masked log-softmax, and finite differences
# --------------------------------------------------------------------------
def test_gradient_against_autograd_masked_log_softmax():
    z, ids = _rand_rows(12, 300, 6, dtype=np.float32)
    rng = np.random.default_rng(7)
    g = rng.standard_normal(len(ids))
    lr = orc.log_rho_f32(1e-2)
    out = orc.rows(z, ids, lr, grad_out=g, want_dz=True, want_flags=True)
    # Def. 5.2 in closed form, row by row: log pi_mp(y) = z_y - log sum_{k in V_S} e^{z_k}, with V_S a fixed
    # index set built here from Def. 5.1 (numpy, independent of the oracle); autograd differentiates that.
    zt = torch.from_numpy(z.astype(np.float64)).requires_grad_(True)
    tau = (z.max(axis=1) + lr).astype(np.float32).astype(np.float64)
    loss = torch.zeros((), dtype=torch.float64)
    rows_with_grad = 0
    for i in range(len(ids)):
        safe = np.nonzero(z[i].astype(np.float64) >= tau[i])[0]
        if ids[i] not in safe:
            continue                                    # probability zero: no term in the objective (Sec. 5.3)
        rows_with_grad += 1
        loss = loss + g[i] * (zt[i, ids[i]] - torch.logsumexp(zt[i, torch.from_numpy(safe)], dim=0))
    assert 0 < rows_with_grad < len(ids)
    loss.backward()
    want = zt.grad.numpy()
    np.testing.assert_allclose(out["dz"], want, rtol=0, atol=1e-12)   # rows with y pruned: all zero


def test_gradient_finite_differences():
    z, ids = _rand_rows(3, 40, 8)
    zf = z.astype(np.float32).astype(np.float64)
    lr = orc.log_rho_f32(1e-1)
    base = orc.rows(zf, ids, lr, want_dz=True, want_flags=True, grad_out=np.ones(3))
    h = 1e-6
    for i in range(3):
        if not base["y_in_safe"][i]:
            ids[i] = int(zf[i].argmax())
    base = orc.rows(zf, ids, lr, want_dz=True, want_flags=True, grad_out=np.ones(3))
    for i in range(3):
        gap = np.abs(zf[i] - base["tau"][i]).min()
        assert gap > 1e-3
        for k in range(40):
            if k == int(zf[i].argmax()):
                continue      # moving the max moves the threshold; the set is held fixed (Sec. 5.5)
            zp = zf.copy(); zp[i, k] += h
            zm = zf.copy(); zm[i, k] -= h
            fp = orc.rows(zp, ids, lr)["logp"][i]
            fm = orc.rows(zm, ids, lr)["logp"][i]
            fd = (fp - fm) / (2 * h)
            assert abs(fd - base["dz"][i, k]) < 1e-8
            if not base["safe_flags"][i, k]:
                assert fd == 0.0


# --------------------------------------------------------------------------
# theory checks on generated train / infer pairs
# --------------------------------------------------------------------------
def test_mismatch_bound_prop_4_2():
    """|Delta_a| <= 2 eps_max (1 - p_a(z_c)) for some z_c on the segment; since
    p_a(z_c) >= p_a exp(-2 eps_max) this gives the checkable bound below, and
    Delta_a = -eps_a + log sum_j p_j exp(eps_j) exactly (Prop. 4.2's setting)."""
    for cfg in (0, 1):
        wl = workloads.make_rows(cfg, n=24, v=3000)
        zt = wl.z_train.to(torch.float64).numpy()
        zi = wl.z_infer.to(torch.float64).numpy()
        ids = wl.ids.numpy()
        lr = orc.log_rho_f32(0.0)
        a = orc.rows(wl.z_train, ids, lr)
        b = orc.rows(wl.z_infer, ids, lr)
        eps = zi - zt
        eps_max = np.abs(eps).max(axis=1)
        delta = a["logp"] - b["logp"]
        r = np.arange(len(ids))
        p = scipy.special.softmax(zt, axis=1)
        exact = -eps[r, ids] + np.log((p * np.exp(eps)).sum(axis=1))
        np.testing.assert_allclose(delta, exact, rtol=0, atol=1e-11)
        bound = 2 * eps_max * (1 - p[r, ids] * np.exp(-2 * eps_max))
        assert np.all(np.abs(delta) <= bound + 1e-12)
        assert np.all(np.abs(delta) <= 2 * eps_max + 1e-12)


def test_bias_bound_prop_5_5_single_step():
    """TV(pi_mp, pi) = 1 - Z exactly, and |E_mp R - E R| <= R_max (1 - Z) (Prop. 5.5, T = 1)."""
    wl = workloads.make_rows(0, n=12, v=5000)
    z = wl.z_train.numpy().astype(np.float64)
    rng = np.random.default_rng(9)
    for rho in (1e-2, 1e-4, math.exp(-13.0)):
        out = orc.rows(wl.z_train, wl.ids.numpy(), orc.log_rho_f32(rho), want_flags=True)
        f = out["safe_flags"].astype(bool)
        pi = scipy.special.softmax(z, axis=1)
        pmp = np.where(f, np.exp(z - out["lse_safe"][:, None]), 0.0)
        one_minus_z = -np.expm1(out["lse_safe"] - out["lse_full"])
        tv = 0.5 * np.abs(pmp - pi).sum(axis=1)
        np.testing.assert_allclose(tv, one_minus_z, rtol=1e-9, atol=1e-14)
        rmax = 1.0
        R = rng.uniform(0, rmax, size=z.shape)
        gap = np.abs((pmp * R).sum(axis=1) - (pi * R).sum(axis=1))
        assert np.all(gap <= rmax * one_minus_z + 1e-14)


# --------------------------------------------------------------------------
# LM-head wrapper: chain rule through the linear map
# --------------------------------------------------------------------------
def test_lmhead_oracle_against_autograd():
    wl = workloads.make_lmhead(n=10, d=32, v=200)
    lr = orc.log_rho_f32(1e-2)
    g = wl.grad_out.numpy().astype(np.float64)
    out = orc.lmhead(wl.hidden, wl.w_train, wl.ids.numpy(), lr, grad_out=g, want_flags=True)
    H = wl.hidden.to(torch.float64).requires_grad_(True)
    W = wl.w_train.to(torch.float64).requires_grad_(True)
    z = H @ W.T
    np.testing.assert_allclose(out["z"], z.detach().numpy(), rtol=0, atol=1e-13)
    z_np = z.detach().numpy()
    tau = (z_np.max(axis=1) + np.float64(lr)).astype(np.float32).astype(np.float64)
    loss = torch.zeros((), dtype=torch.float64)
    for i in range(10):                                 # Def. 5.2 in closed form over the fixed index set of Def. 5.1
        safe = np.nonzero(z_np[i] >= tau[i])[0]
        y = int(wl.ids[i])
        assert (y in safe) == bool(out["y_in_safe"][i])
        if y not in safe:
            continue
        lp_i = z[i, y] - torch.logsumexp(z[i, torch.from_numpy(safe)], dim=0)
        assert abs(out["logp"][i] - lp_i.item()) <= 1e-12
        loss = loss + g[i] * lp_i
    loss.backward()
    np.testing.assert_allclose(out["d_hidden"], H.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["d_w"], W.grad.numpy(), rtol=0, atol=1e-12)


def test_threads_do_not_change_results():
    wl = workloads.make_rows(1, n=13, v=2000)
    g = wl.grad_out.numpy().astype(np.float64)
    a = orc.rows(wl.z_train, wl.ids.numpy(), orc.log_rho_f32(1e-4), grad_out=g, want_dz=True, threads=1)
    b = orc.rows(wl.z_train, wl.ids.numpy(), orc.log_rho_f32(1e-4), grad_out=g, want_dz=True, threads=4)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


# --------------------------------------------------------------------------
# sequence level: importance weights, cumulative mismatch, token veto
# (Thm. 4.1; App. A protocol items 4 and 5)
# --------------------------------------------------------------------------
def _veto_constant():
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            if line.startswith("veto_threshold_appA"):
                return float(line.split()[1])
    raise AssertionError("fixture line missing")


def test_sequence_hand_example():
    """Two short sequences worked by hand: weights are e^(lt - li), the
    sequence mismatch is their log-product, and 1e-4 (App. A item 5) vetoes."""
    thr = _veto_constant()
    assert thr == 1e-4
    lt = np.log(np.array([0.5, 0.25, 0.2, 0.5, 1e-6], np.float64)).astype(np.float32)
    li = np.log(np.array([0.25, 0.5, 0.2, 0.5, 0.5], np.float64)).astype(np.float32)
    out = orc.sequences(lt, li, [0, 3, 5], orc.log_threshold_f32(thr))
    np.testing.assert_allclose(out["weight"], [2.0, 0.5, 1.0, 1.0, 2e-6], rtol=2e-6)
    np.testing.assert_allclose(out["seq_log_ratio"], [0.0, math.log(2e-6)], atol=1e-6)
    np.testing.assert_allclose(out["seq_min_weight"], [0.5, 2e-6], rtol=2e-6)
    assert out["seq_veto"].tolist() == [0, 1]


def test_sequence_weights_against_numpy_and_identities():
    rng = np.random.default_rng(5)
    n, n_seq = 5000, 37
    lt = (-3.0 * rng.random(n)).astype(np.float32)
    li = (lt + 0.05 * rng.standard_normal(n)).astype(np.float32)
    cuts = np.sort(rng.choice(np.arange(1, n), n_seq - 1, replace=False))
    off = np.concatenate([[0], cuts, [n]])
    out = orc.sequences(lt, li, off, orc.log_threshold_f32(1e-4))
    l = lt.astype(np.float64) - li.astype(np.float64)
    np.testing.assert_allclose(out["weight"], np.exp(l), rtol=1e-14)
    for s in range(n_seq):
        seg = slice(off[s], off[s + 1])
        assert abs(out["seq_log_ratio"][s] - math.fsum(l[seg])) <= 1e-12
        # the sequence weight is the product of the token weights (Thm. 4.1's e^{Delta_y})
        assert abs(math.exp(out["seq_log_ratio"][s]) - np.prod(out["weight"][seg])) <= 1e-9 * np.prod(out["weight"][seg])
        assert out["seq_min_weight"][s] == out["weight"][seg].min()
    assert not out["seq_veto"].any()
    # identical engines: every weight 1, no mismatch
    same = orc.sequences(lt, lt, off, orc.log_threshold_f32(1e-4))
    assert np.all(same["weight"] == 1.0) and np.all(same["seq_log_ratio"] == 0.0)


def test_sequence_veto_boundary_and_conventions():
    lthr = orc.log_threshold_f32(1e-4)
    base = np.float32(-1.0)
    # a token exactly at the threshold is kept (item 5 says "<"), one fp32 step below is vetoed
    at = np.float32(base + lthr)
    assert np.float32(at - base) == lthr
    below = np.nextafter(at, np.float32(-np.inf))
    out = orc.sequences([at, below], [base, base], [0, 1, 2], lthr)
    assert out["seq_veto"].tolist() == [0, 1]
    # a pruned sampled token under the training policy: weight zero (Sec. 5.3), sequence discarded
    out = orc.sequences([-np.inf, -0.5, -np.inf], [-0.7, -0.5, -np.inf], [0, 2, 3], lthr)
    assert out["weight"].tolist() == [0.0, 1.0, 0.0]
    assert out["seq_log_ratio"].tolist() == [-np.inf, -np.inf] and out["seq_veto"].tolist() == [1, 1]
    # undefined or infinite weights discard the sequence too; an empty sequence is kept
    out = orc.sequences([np.nan, -0.5, -0.1], [-0.5, -np.inf, -0.1], [0, 1, 2, 2, 3], lthr)
    assert np.isnan(out["weight"][0]) and out["weight"][1] == np.inf
    assert out["seq_veto"].tolist() == [1, 1, 0, 0]
    assert out["seq_min_weight"][2] == np.inf and out["seq_log_ratio"][2] == 0.0
    # tokens owned by no sequence are not written
    out = orc.sequences([-1.0, -1.0, -1.0], [-1.0, -1.0, -1.0], [1, 2], lthr)
    assert np.isnan(out["weight"][0]) and out["weight"][1] == 1.0 and np.isnan(out["weight"][2])


def test_sequence_weight_is_the_change_of_measure_of_thm_4_1():
    """Thm. 4.1's step: an expectation under the inference policy equals the
    expectation under the training policy of e^{-Delta_y} f(y).  Enumerate every
    two-token sequence of a 5-token vocabulary; Delta_y comes from the oracle."""
    rng = np.random.default_rng(9)
    v = 5
    zt = rng.standard_normal((1 + v, v))          # step-1 logits, then step-2 logits per first token
    zi = zt + 0.3 * rng.standard_normal(zt.shape)
    lpt = torch.log_softmax(torch.from_numpy(zt), -1).numpy()
    lpi = torch.log_softmax(torch.from_numpy(zi), -1).numpy()
    f = rng.standard_normal((v, v))
    lt, li, off = [], [], [0]
    for a in range(v):
        for b in range(v):
            lt += [lpt[0, a], lpt[1 + a, b]]
            li += [lpi[0, a], lpi[1 + a, b]]
            off.append(len(lt))
    out = orc.sequences(np.array(lt, np.float32), np.array(li, np.float32), off, orc.log_threshold_f32(1e-4))
    p_train = np.exp(np.array(lt).reshape(-1, 2).sum(1))
    p_infer = np.exp(np.array(li).reshape(-1, 2).sum(1))
    lhs = float((p_infer * f.ravel()).sum())
    rhs = float((p_train * np.exp(-out["seq_log_ratio"]) * f.ravel()).sum())
    assert abs(lhs - rhs) <= 1e-6
    assert abs(p_train.sum() - 1.0) <= 1e-12 and abs(p_infer.sum() - 1.0) <= 1e-12


# ---------------------------------------------------------------------------
# entropy of the constrained policy
# ---------------------------------------------------------------------------
def test_entropy_against_scipy_and_closed_forms():
    import scipy.stats
    z, ids = _rand_rows(12, 700, 31)
    lr = orc.log_rho_f32(1e-2)
    out = orc.rows(z, ids, lr, want_entropy=True, want_flags=True)
    for i in range(z.shape[0]):
        keep = z[i] >= np.float64(np.float32(z[i].max() + np.float64(lr)))       # mask rebuilt here
        np.testing.assert_array_equal(keep, out["safe_flags"][i] == 1)
        p = np.exp(z[i][keep] - z[i].max())
        want = scipy.stats.entropy(p / p.sum())
        assert abs(out["entropy"][i] - want) <= 1e-12
        assert -1e-15 <= out["entropy"][i] <= math.log(keep.sum()) + 1e-12
        # H = lse_safe - E_pi[z]
        pi = p / p.sum()
        assert abs(out["entropy"][i] - (out["lse_safe"][i] - (pi * z[i][keep]).sum())) <= 1e-10
    # closed forms: c equal logits above the threshold -> log c; a lone maximum -> 0
    zz = np.full((1, 50), -100.0); zz[0, :7] = 3.25
    assert abs(orc.rows(zz, [0], lr, want_entropy=True)["entropy"][0] - math.log(7)) <= 1e-14
    zz[0, 1:] = -100.0
    assert orc.rows(zz, [0], lr, want_entropy=True)["entropy"][0] == 0.0
    # no pruning: the entropy of the plain softmax
    full = orc.rows(z, ids, orc.log_rho_f32(0.0), want_entropy=True)["entropy"]
    np.testing.assert_allclose(full, [scipy.stats.entropy(scipy.special.softmax(r)) for r in z], rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# the finite-mask variant (Sec. 5.5 "Logit Masking Strategy", App. A item 3)
# ---------------------------------------------------------------------------
def _torch_finite_mask(z, ids, rho, mask_value, g):
    """The variant from its closed form, row by row.  Every pruned logit counts as the constant `mask_value`
    (Sec. 5.5), so with K the kept index set, decided in the tensor's own dtype (App. A item 3),
        lse = log( sum_{k in K} e^{z_k} + (V - |K|) e^{mask_value} ),
        log-prob of y = (z_y if y in K else mask_value) - lse,
    evaluated in float64 and differentiated by autograd.  Returns (pruned flags, thresholds, log-probs, gradient)."""
    n, v = z.shape
    zz = z.clone().to(torch.float64).requires_grad_(True)
    top = z.amax(dim=1)
    if z.dtype == torch.bfloat16:
        # On the GPU, where the method runs, torch adds a Python scalar to a bf16 tensor in fp32 and
        # rounds the sum; its CPU kernel rounds the scalar to bf16 first (observed: 8.375 + log(0.01)
        # gives 3.78125 instead of 3.765625).  The GPU behaviour is the one followed, written out
        # here; tests/test_gpu_finite_mask.py checks it against torch's own GPU add.
        thr = (top.float() + torch.tensor(math.log(rho), dtype=torch.float32)).to(torch.bfloat16)
    else:
        thr = top + math.log(rho)
    kept = z >= thr[:, None]                            # comparison in the storage dtype
    picked = []
    for i in range(n):
        idx = torch.nonzero(kept[i]).flatten()
        const = torch.full((v - idx.numel(),), float(mask_value), dtype=torch.float64)
        lse = torch.logsumexp(torch.cat([zz[i, idx], const]), dim=0)
        y = int(ids[i])
        picked.append((zz[i, y] if bool(kept[i, y]) else torch.tensor(float(mask_value), dtype=torch.float64)) - lse)
    picked = torch.stack(picked)
    (picked * torch.as_tensor(g, dtype=torch.float64)).sum().backward()
    return (~kept).numpy(), thr.to(torch.float64).numpy(), picked.detach().numpy(), zz.grad.numpy()


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32, torch.bfloat16])
def test_finite_mask_against_torch(dtype):
    gen = torch.Generator().manual_seed(77)
    z = (3.0 * torch.randn(16, 900, generator=gen, dtype=torch.float64)).to(dtype)
    ids = torch.randint(0, 900, (16,), generator=gen).numpy()
    ids[0] = int(z[0].argmin())                     # a pruned sampled token
    ids[1] = int(z[1].argmax())
    g = torch.randn(16, generator=gen, dtype=torch.float64).numpy()
    for rho, mask_value in ((1e-2, -50.0), (math.exp(-13.0), -50.0), (1e-1, -7.5)):
        pruned, thr, lp, grad = _torch_finite_mask(z, ids, rho, mask_value, g)
        out = orc.rows_finite_mask(z, ids, math.log(rho), mask_value, grad_out=g, want_flags=True, want_dz=True)
        np.testing.assert_array_equal(out["safe_flags"] == 0, pruned)
        np.testing.assert_array_equal(out["tau"], thr)
        np.testing.assert_allclose(out["logp"], lp, rtol=0, atol=1e-11)
        # autograd hands the gradient back in the leaf's dtype: one rounding to that type
        eps = {torch.float64: 0.0, torch.float32: 2.0 ** -24, torch.bfloat16: 2.0 ** -8}[dtype]
        assert np.all(np.abs(out["dz"] - grad) <= eps * np.abs(out["dz"]) + 1e-12)
        np.testing.assert_array_equal((out["dz"] == 0), (grad == 0))
        np.testing.assert_array_equal(out["safe_count"], (~pruned).sum(1))
        np.testing.assert_array_equal(out["y_in_safe"], ~pruned[np.arange(16), ids])
    assert out["y_in_safe"][0] == 0 and np.isfinite(out["logp"][0])
    assert np.abs(out["dz"][0]).max() > 0           # a pruned sampled token still pulls the safe logits down


def test_finite_mask_threshold_is_rounded_to_the_logits_dtype():
    """bf16 logits: the threshold 10 + log(1e-4) = 0.78966 is rounded to the bf16 grid point 0.7890625,
    which then counts as safe; the exact rule (one fp32 threshold, Def. 5.1) prunes it.  The variant
    reproduces that artefact, the main oracle does not."""
    row = torch.tensor([[10.0, 0.7890625, 0.79296875, 0.78515625, -3.0]], dtype=torch.bfloat16)
    lit = orc.rows_finite_mask(row, [0], math.log(1e-4), want_flags=True)
    np.testing.assert_array_equal(lit["safe_flags"][0], [1, 1, 1, 0, 0])
    assert lit["tau"][0] == 0.7890625
    exact = orc.rows(row, [0], orc.log_rho_f32(1e-4), want_flags=True)
    np.testing.assert_array_equal(exact["safe_flags"][0], [1, 0, 1, 0, 0])
    pruned, thr, _, _ = _torch_finite_mask(row, [0], 1e-4, -50.0, [1.0])
    np.testing.assert_array_equal(pruned[0], [False, False, False, True, True])
    # fp32 logits: both rules agree
    row32 = row.to(torch.float32)
    np.testing.assert_array_equal(orc.rows_finite_mask(row32, [0], math.log(1e-4), want_flags=True)["safe_flags"],
                                  orc.rows(row32, [0], orc.log_rho_f32(1e-4), want_flags=True)["safe_flags"])


def test_finite_mask_converges_to_the_exact_rule():
    """With the mask far below the row the pruned tokens' mass vanishes: log-probs and gradients of rows
    whose sampled token is safe equal the exact -inf semantics (Prop. 5.6)."""
    z, ids = _rand_rows(10, 400, 5)
    ids = z.argmax(1)
    g = np.linspace(-1, 1, 10)
    lit = orc.rows_finite_mask(z, ids, math.log(1e-2), -745.0, grad_out=g, want_dz=True)
    # fp64 logits: the exact oracle rounds its threshold to fp32, so compare away from the boundary
    ex = orc.rows(z, ids, orc.log_rho_f32(1e-2), grad_out=g, want_dz=True, band=1e-5)
    ok = ex["band_count"] == 0
    assert ok.sum() >= 8
    np.testing.assert_allclose(lit["logp"][ok], ex["logp"][ok], rtol=0, atol=1e-12)
    np.testing.assert_allclose(lit["dz"][ok], ex["dz"][ok], rtol=0, atol=1e-12)
    # a mask within reach shows the pruned tokens' mass: logp drops by log(1 + (V - c) e^{mask - lse});
    # with the paper's -50 that is ~1e-24, below what a double can show next to an O(1) log-prob
    lit5 = orc.rows_finite_mask(z, ids, math.log(1e-2), -5.0)
    extra = (400 - ex["safe_count"]) * np.exp(-5.0 - ex["lse_safe"])
    assert extra[ok].min() > 1e-5
    np.testing.assert_allclose((ex["logp"] - lit5["logp"])[ok], np.log1p(extra)[ok], rtol=1e-9, atol=1e-13)
    lit50 = orc.rows_finite_mask(z, ids, math.log(1e-2), -50.0)
    np.testing.assert_allclose(lit50["logp"][ok], ex["logp"][ok], rtol=0, atol=1e-15)
