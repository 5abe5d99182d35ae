"""GPU parity of the finite-mask variant (Sec. 5.5 "Logit Masking Strategy", App. A item 3) and of the
entropy output, against the fp64 oracle, through the C ABI.

Finite-mask variant: membership, sizes and flags are exact (the threshold is the fp32 sum rounded to
the logits' storage type on both sides); lse / logp to 1e-5 (fp32 logits) or 2e-3 (bf16); the gradient
to the same per-element bound as the exact rule.  The reading "threshold as a GPU evaluates a
tensor-plus-scalar add" is checked here against torch's own GPU add.
Entropy: |H_gpu - H_oracle| <= 1e-5 * max(1, log V) for fp32 logits, 2e-3 for bf16 (fp32 sums of exactly
widened inputs; the bf16 figure is the path's general tolerance, the error observed is ~1e-6).
"""
import math

import numpy as np
import pytest
import torch

from oracle import dvp_oracle as orc
from paper_2512_23087_amd import workloads
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


def _case(n, v, dtype, seed, scale=3.0):
    g = torch.Generator().manual_seed(seed)
    zt = (scale * torch.randn(n, v, generator=g)).to(dtype)
    zi = (zt.float() + 0.05 * torch.randn(n, v, generator=g)).to(dtype)
    ids = torch.randint(0, v, (n,), generator=g)
    ids[0] = int(zt[0].float().argmin())          # a pruned sampled token
    ids[1] = int(zt[1].float().argmax())
    gout = torch.randn(n, generator=g)
    return zt.cuda(), zi.cuda(), ids.cuda(), gout.cuda()


def _check_finite(dvp, zt, zi, ids, gout, rho, mask_value, split_backward=False):
    lr = dvp.log_rho(rho)
    tol = parity.TOL[zt.dtype]
    n, v = zt.shape
    if split_backward:
        res = dvp.dvp_forward(zt, zi, ids, lr, safe_bits=True, mask_value=mask_value)
        dz = dvp.dvp_backward(zt, ids, gout, res.train.row_max, res.train.lse_safe, res.row_flags, lr,
                              mask_value=mask_value)
    else:
        res = dvp.dvp_forward_backward(zt, zi, ids, gout, lr, safe_bits=True, lse_full=True, mask_value=mask_value)
        dz = res.dz
    torch.cuda.synchronize()
    idh = ids.cpu().numpy()
    g = gout.cpu().numpy().astype(np.float64)
    flags = res.row_flags.cpu().numpy()
    for name, side, z, bit in (("train", res.train, zt, 1), ("infer", res.infer, zi, 2)):
        o = orc.rows_finite_mask(z.cpu(), idh, float(lr), mask_value, grad_out=g, want_flags=True,
                                 want_dz=(name == "train"))
        np.testing.assert_array_equal(side.row_max.cpu().double().numpy(), o["row_max"], err_msg=name)
        np.testing.assert_array_equal(side.safe_count.cpu().numpy(), o["safe_count"], err_msg=name)
        np.testing.assert_array_equal(side.flags_matrix(v).cpu().numpy(), o["safe_flags"], err_msg=name)
        assert np.abs(side.lse_safe.cpu().double().numpy() - o["lse"]).max() <= tol, name
        lp = side.logp.cpu().double().numpy()
        assert np.isfinite(lp).all()
        assert np.abs(lp - o["logp"]).max() <= tol, name
        np.testing.assert_array_equal((flags & bit) != 0, o["y_in_safe"] == 1)
        if name == "train":
            got = dz.cpu().double().numpy()
            scale = np.maximum(1.0, np.abs(g))[:, None]
            if dz.dtype == torch.bfloat16:
                mag = np.abs(o["dz"])
                half_ulp = np.where(mag > 0, np.exp2(np.floor(np.log2(np.maximum(mag, 1e-300))) - 8), 0.0)
                bound = np.maximum(tol, half_ulp + 1e-5 * scale)
            else:
                bound = tol * scale
            assert (np.abs(got - o["dz"]) / bound).max() <= 1.0
            assert np.all(got[o["safe_flags"] == 0] == 0.0)
            ot = o
    return res, ot


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("v", [5, 1001, 32000])
def test_finite_mask_against_oracle(dvp, dtype, v):
    zt, zi, ids, gout = _case(7, v, dtype, seed=v)
    for rho, mask in ((1e-2, -50.0), (math.exp(-13.0), -50.0), (1e-1, -7.5)):
        res, ot = _check_finite(dvp, zt, zi, ids, gout, rho, mask)
        _check_finite(dvp, zt, zi, ids, gout, rho, mask, split_backward=True)
    if v > 100:
        assert ot["y_in_safe"][0] == 0 and np.abs(ot["dz"][0]).max() > 0
        assert res.dz[0].float().abs().max().item() > 0     # a pruned sampled token still moves the safe logits


def test_threshold_rounding_matches_a_gpu_tensor_plus_scalar_add(dvp):
    """bf16 logits: the variant's threshold is what torch's GPU kernel returns for `max + log(rho)` on
    a bf16 tensor, and membership is `not (z < that)`: compared token by token, on rows that contain
    every bf16 grid point around the threshold."""
    g = torch.Generator().manual_seed(3)
    n, v = 64, 4096
    z = (4.0 * torch.randn(n, v, generator=g)).to(torch.bfloat16)
    for i in range(n):                              # plant the grid points next to each row's threshold
        m = z[i].float().max().item()
        t = torch.tensor(m + math.log(1e-2), dtype=torch.float32).to(torch.bfloat16)
        bits = t.view(torch.int16).item()
        z[i, 1:8] = torch.tensor([bits + d for d in (-3, -2, -1, 0, 1, 2, 3)], dtype=torch.int16).view(torch.bfloat16)
    z = z.cuda()
    ids = torch.zeros(n, dtype=torch.int64, device="cuda")
    rho = 1e-2
    thr = z.max(dim=-1, keepdim=True).values + math.log(rho)          # torch's GPU add, bf16 result
    assert thr.dtype == torch.bfloat16
    want_safe = ~(z < thr)
    res = dvp.dvp_forward(z, None, ids, dvp.log_rho(rho), safe_bits=True, mask_value=-50.0)
    torch.cuda.synchronize()
    got_safe = res.train.flags_matrix(v).bool()
    assert torch.equal(got_safe, want_safe)
    o = orc.rows_finite_mask(z.cpu(), ids.cpu().numpy(), float(dvp.log_rho(rho)), -50.0, want_flags=True)
    np.testing.assert_array_equal(o["tau"], thr.double().squeeze(1).cpu().numpy())
    # the exact rule differs on some of these rows: it never admits a token below the fp32 threshold
    exact = dvp.dvp_forward(z, None, ids, dvp.log_rho(rho), safe_bits=True)
    torch.cuda.synchronize()
    diff = (exact.train.safe_count != res.train.safe_count).sum().item()
    assert diff > 0


def test_finite_mask_is_refused_where_it_is_not_defined(dvp):
    zt, zi, ids, gout = _case(4, 64, torch.bfloat16, seed=1)
    lr = dvp.log_rho(1e-2)
    with pytest.raises(dvp.DvpError) as e:
        dvp.dvp_forward(zt, zi, ids, lr, entropy=True, mask_value=-50.0)
    assert e.value.status == 5
    with pytest.raises(dvp.DvpError) as e:
        dvp.dvp_forward(zt, zi.float().to(torch.float8_e4m3fn), ids, lr, mask_value=-50.0)
    assert e.value.status == 3


# ---------------------------------------------------------------------------
# entropy of the constrained policy
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("v,aligned", [(5, True), (1001, False), (4096, True), (32000, True), (151936, True)])
def test_entropy_against_oracle(dvp, dtype, v, aligned):
    n = 6
    zt, zi, ids, gout = _case(n, v, dtype, seed=100 + v, scale=2.0)
    if not aligned:                                  # odd offset: the re-reading kernel
        store = torch.zeros(n, v + 3, dtype=dtype, device="cuda")
        store[:, 1:v + 1] = zt
        zt = store[:, 1:v + 1]
    tol = 1e-5 * max(1.0, math.log(v)) if dtype == torch.float32 else 2e-3
    for rho in (1e-2, 1e-4, 0.0):
        lr = dvp.log_rho(rho)
        res = dvp.dvp_forward_backward(zt, zi, ids, gout, lr, entropy=True)
        ref = dvp.dvp_forward_backward(zt, zi, ids, gout, lr)
        torch.cuda.synchronize()
        for side, z in ((res.train, zt), (res.infer, zi)):
            o = orc.rows(z.cpu().contiguous(), ids.cpu().numpy(), np.float32(lr), want_entropy=True, threads=4)
            got = side.entropy.cpu().double().numpy()
            assert np.abs(got - o["entropy"]).max() <= tol
            assert np.all(got >= -tol) and np.all(got <= np.log(o["safe_count"]) + tol)
        # asking for the entropy changes nothing else
        assert torch.equal(res.train.safe_count, ref.train.safe_count)
        assert (res.train.logp - ref.train.logp).abs().nan_to_num(0.0).max().item() <= 1e-6
        assert torch.equal(res.dz, ref.dz)


def test_entropy_with_byte_inference_logits(dvp):
    zt, zi, ids, gout = _case(8, 32000, torch.bfloat16, seed=9)
    zi8 = workloads.through_e4m3(zi.float()).to(torch.float8_e4m3fn)
    lr = dvp.log_rho(1e-3)
    res = dvp.dvp_forward(zt, zi8, ids, lr, entropy=True)
    torch.cuda.synchronize()
    o = orc.rows(zi8.view(torch.uint8).cpu(), ids.cpu().numpy(), np.float32(lr), want_entropy=True)
    assert np.abs(res.infer.entropy.cpu().double().numpy() - o["entropy"]).max() <= 1e-5 * math.log(32000)
