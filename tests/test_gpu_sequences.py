"""GPU parity of dvp_sequence_weights against the fp64 oracle, through the C ABI.

Bars: the veto flag is bit-exact (both sides decide on the fp32 difference of
the two log-probabilities against the same fp32 constant); weights agree to a
relative 4e-6 (one fp32 rounding of the difference, amplified by its magnitude,
plus the fp32 exponential); the sequence mismatch is summed in double on the
GPU and stored as fp32: 1e-6 * max(1, |Delta|) + the fp32 rounding of the
per-token differences, n * 2^-24 * max|l| at worst, bounded here by 1e-6 * sum|l|.
"""
import math

import numpy as np
import pytest
import torch

from oracle import dvp_oracle as orc
from paper_2512_23087_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


def _check(dvp, lt, li, off, thr=1e-4):
    lthr = dvp.log_threshold(thr)
    assert np.float32(lthr) == orc.log_threshold_f32(thr)
    res = dvp.dvp_sequence_weights(lt, li, off, lthr)
    torch.cuda.synchronize()
    o = orc.sequences(lt.cpu().numpy(), li.cpu().numpy(), off.cpu().numpy(), np.float32(lthr))
    np.testing.assert_array_equal(res.seq_veto.cpu().numpy(), o["seq_veto"])
    offs = off.cpu().numpy()
    owned = np.zeros(lt.shape[0], bool)
    for s in range(len(offs) - 1):
        owned[offs[s]:offs[s + 1]] = True
    w = res.weight.cpu().double().numpy()[owned]
    wo = o["weight"][owned]
    l = (lt.cpu().double() - li.cpu().double()).numpy()[owned]
    fin = np.isfinite(wo)
    np.testing.assert_array_equal(np.isnan(w), np.isnan(wo))
    np.testing.assert_array_equal(w[~fin & ~np.isnan(wo)], wo[~fin & ~np.isnan(wo)])
    rel = np.abs(w[fin] - wo[fin]) / np.maximum(wo[fin], 1e-30)
    lim = 4e-6 + 2.0 ** -23 * np.abs(np.where(np.isfinite(l[fin]), l[fin], 0.0))
    assert np.all(rel <= lim), "weight off by %.2e relative" % rel.max()
    d = res.seq_log_ratio.cpu().double().numpy()
    mn = res.seq_min_weight.cpu().double().numpy()
    for s in range(len(offs) - 1):
        ls = (lt.cpu().double() - li.cpu().double()).numpy()[offs[s]:offs[s + 1]]
        ref = o["seq_log_ratio"][s]
        if np.isfinite(ref):
            tol = 1e-6 * max(1.0, abs(ref)) + 1e-6 * np.abs(ls[np.isfinite(ls)]).sum()
            assert abs(d[s] - ref) <= tol, (s, d[s], ref)
        else:
            assert (np.isnan(d[s]) and np.isnan(ref)) or d[s] == ref
        mo = o["seq_min_weight"][s]
        if np.isfinite(mo):
            assert abs(mn[s] - mo) <= 1e-5 * max(mo, 1e-30)
        else:
            assert (np.isnan(mn[s]) and np.isnan(mo)) or mn[s] == mo
    return res, o


def test_weights_from_the_row_path_outputs(dvp):
    """End to end on configs[1]-shaped logits: log-probs from dvp_forward feed the sequence step."""
    wl = workloads.make_rows(1, device="cuda", n=2048, v=32000)
    r = dvp.dvp_forward(wl.z_train, wl.z_infer, wl.ids, dvp.log_rho(1e-4))
    off = torch.tensor([0, 1, 130, 130, 900, 2048], dtype=torch.int64, device="cuda")
    res, o = _check(dvp, r.train.logp, r.infer.logp, off)
    # e4m3-rounded inference logits: some sampled tokens are pruned on one side only
    assert o["seq_veto"].sum() >= 1


def test_long_sequences_and_ragged_batch(dvp):
    """32 sequences with the paper's 16384-token limit (Sec. 6), ragged lengths, small mismatch."""
    g = torch.Generator(device="cuda"); g.manual_seed(0xD5B0 + 7)
    lens = torch.randint(1, 16385, (32,), generator=g, device="cuda")
    lens[3] = 16384; lens[4] = 1
    off = torch.cat([torch.zeros(1, dtype=torch.int64, device="cuda"), torch.cumsum(lens, 0)])
    n = int(off[-1].item())
    lt = -3.0 * torch.rand(n, generator=g, device="cuda")
    li = lt + 0.02 * torch.randn(n, generator=g, device="cuda")
    li[100] = lt[100] + 12.0           # one catastrophic token: weight e^-12 < 1e-4
    res, o = _check(dvp, lt, li, off)
    seq_of_100 = int(np.searchsorted(off.cpu().numpy(), 100, side="right") - 1)
    assert o["seq_veto"][seq_of_100] == 1 and o["seq_veto"].sum() == 1


def test_veto_boundary_infinities_and_empty(dvp):
    lthr = np.float32(dvp.log_threshold(1e-4))
    base = np.float32(-1.0)
    at = np.float32(base + lthr)
    below = np.nextafter(at, np.float32(-np.inf))
    lt = torch.tensor([at, below, -np.inf, -0.5, -np.inf, np.nan, -0.5, -0.1], dtype=torch.float32, device="cuda")
    li = torch.tensor([base, base, -0.7, -0.5, -np.inf, -0.5, -np.inf, -0.1], dtype=torch.float32, device="cuda")
    off = torch.tensor([0, 1, 2, 4, 5, 6, 7, 7, 8], dtype=torch.int64, device="cuda")
    res, o = _check(dvp, lt, li, off)
    assert res.seq_veto.cpu().tolist() == [0, 1, 1, 1, 1, 1, 0, 0]
    # unowned tokens are left alone; offsets outside [0, N) are ignored, not dereferenced
    w = torch.full((8,), -7.0, device="cuda")
    off2 = torch.tensor([-5, 2, 6], dtype=torch.int64, device="cuda")
    r2 = dvp.dvp_sequence_weights(lt, li, off2, float(lthr), weight=w)
    off3 = torch.tensor([6, 100], dtype=torch.int64, device="cuda")
    r3 = dvp.dvp_sequence_weights(lt, li, off3, float(lthr))
    torch.cuda.synchronize()
    assert r2.weight[6:].cpu().tolist() == [-7.0, -7.0] and abs(r2.weight[0].item() - 1e-4) < 1e-9
    assert r2.seq_veto.cpu().tolist() == [1, 1] and r3.seq_veto.cpu().tolist() == [1]
    # zero sequences
    r4 = dvp.dvp_sequence_weights(lt, li, torch.zeros(1, dtype=torch.int64, device="cuda"), float(lthr))
    assert r4.seq_veto.numel() == 0


def test_repeated_runs_are_bit_identical(dvp):
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    n = 200000
    lt = -5.0 * torch.rand(n, generator=g, device="cuda")
    li = lt + 0.1 * torch.randn(n, generator=g, device="cuda")
    off = torch.tensor([0, 70000, 70001, 200000], dtype=torch.int64, device="cuda")
    a = dvp.dvp_sequence_weights(lt, li, off, dvp.log_threshold(1e-4))
    b = dvp.dvp_sequence_weights(lt, li, off, dvp.log_threshold(1e-4))
    torch.cuda.synchronize()
    assert torch.equal(a.seq_log_ratio, b.seq_log_ratio) and torch.equal(a.weight, b.weight)
