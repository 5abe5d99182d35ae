"""GPU parity of the row path (dvp_forward / dvp_backward / dvp_forward_backward)
against the fp64 oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

from paper_2512_23087_amd import workloads
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


@pytest.fixture(autouse=True, scope="module")
def _small_gradients_in_two_steps_too(dvp):
    # the test matrices are far below the size from which the gradient is written in two steps: force that
    # way for the module (tests that take `gradient_steps` run both ways, the full-size ones the default)
    old = dvp.set_split_min_bytes(0)
    yield
    dvp.set_split_min_bytes(old)


def _run_case(dvp, wl, rho, *, backward, lse_full=True, bits=True, rows=None, threads=8):
    lr = dvp.log_rho(rho)
    assert lr == float(parity.orc.log_rho_f32(rho))      # one shared fp32 constant
    tol = parity.TOL[wl.z_train.dtype]
    v = wl.z_train.shape[1]
    if backward:
        res = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr,
                                       lse_full=lse_full, safe_bits=bits)
    else:
        res = dvp.dvp_forward(wl.z_train, wl.z_infer, wl.ids, lr, lse_full=lse_full, safe_bits=bits)
    torch.cuda.synchronize()
    if rows is None:
        zt, zi = wl.z_train.cpu(), wl.z_infer.cpu()
    else:   # bring back only the sampled rows, keep row numbering via a dense copy
        idx = torch.as_tensor(rows, device=wl.z_train.device)
        zt, zi = wl.z_train[idx].cpu(), wl.z_infer[idx].cpu()
    ids = wl.ids.cpu()
    stats = {}
    if rows is None:
        st = parity.check_side("train", res.train, zt, ids, lr, tol, v, threads=threads)
        si = parity.check_side("infer", res.infer, zi, ids, lr, tol, v, threads=threads)
        parity.check_flags(res.row_flags, st["y_in_safe"], si["y_in_safe"], ids, v, train_safe_count=st["safe_count"])
        if backward:
            stats.update(parity.check_gradient("dz", res.dz, zt, ids, wl.grad_out.cpu(), lr, tol,
                                               threads=threads))
    else:
        sub = _Subset(res, rows)
        ids_s = ids[torch.as_tensor(rows)]
        st = parity.check_side("train", sub.train, zt, ids_s, lr, tol, v, threads=threads)
        si = parity.check_side("infer", sub.infer, zi, ids_s, lr, tol, v, threads=threads)
        parity.check_flags(sub.row_flags, st["y_in_safe"], si["y_in_safe"], ids_s, v, train_safe_count=st["safe_count"])
        if backward:
            stats.update(parity.check_gradient("dz", sub.dz, zt, ids_s,
                                               wl.grad_out.cpu()[torch.as_tensor(rows)], lr, tol,
                                               threads=threads))
    stats.update(train=st, infer=si, result=res)
    return stats


class _Subset:
    """View of a RowResult restricted to some rows (keeps the oracle's work bounded)."""

    def __init__(self, res, rows):
        idx = torch.as_tensor(rows, device=res.row_flags.device)

        class Side:
            pass

        def cut(side):
            s = Side()
            for k in ("logp", "row_max", "lse_safe", "lse_full", "safe_count", "safe_bits"):
                t = getattr(side, k)
                setattr(s, k, None if t is None else t[idx])
            s.flags_matrix = lambda vocab, s=s: type(side).flags_matrix(s, vocab)
            return s

        self.train, self.infer = cut(res.train), cut(res.infer)
        self.row_flags = res.row_flags[idx]
        self.dz = None if res.dz is None else res.dz[idx]


# ---------------------------------------------------------------------------
# the five workload recipes at sizes the oracle finishes in seconds
# ---------------------------------------------------------------------------
def test_config0_fp32_forward_full_size(dvp):
    wl = workloads.make_rows(0, device="cuda")
    st = _run_case(dvp, wl, 1e-4, backward=False)
    assert st["train"]["safe_count"].min() > 100     # the spike recipe keeps thousands of tokens


def test_config1_bf16_forward_backward(dvp, gradient_steps):
    wl = workloads.make_rows(1, device="cuda", n=192)
    st = _run_case(dvp, wl, 1e-4, backward=True)
    assert st["err_grad"] <= 1.0


@pytest.mark.parametrize("rho", [1e-4, math.exp(-13.0)])
def test_config2_heavy_tail_large_vocab(dvp, rho, gradient_steps):
    wl = workloads.make_rows(2, device="cuda", n=80)
    st = _run_case(dvp, wl, rho, backward=True)
    # rows with a uniformly drawn token: (nearly) all outside the safe set, gradient row zero
    forced = wl.forced_rows.cpu().numpy()
    assert (st["train"]["y_in_safe"][forced] == 0).sum() >= forced.sum() - 1
    assert (st["train"]["y_in_safe"][~forced] == 1).sum() > 0


@pytest.mark.parametrize("rho", [1e-2, 1e-4, 1e-6, 0.0])
def test_config3_threshold_sweep(dvp, rho, gradient_steps):
    wl = workloads.make_rows(3, device="cuda", n=48)
    st = _run_case(dvp, wl, rho, backward=True)
    if rho == 0.0:
        v = wl.z_train.shape[1]
        assert np.all(st["train"]["safe_count"] == v)
        res = st["result"]
        assert torch.equal(res.train.lse_safe, res.train.lse_full)   # same sum, same order


# ---------------------------------------------------------------------------
# shapes: ragged tails, tiny vocabularies, both kernels, both dtypes
# ---------------------------------------------------------------------------
def _random_case(n, v, dtype, seed, device="cuda", ld=None, offset=0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    ld = ld or v
    store_t = torch.full((n, ld + offset), float("nan")).to(dtype)
    store_i = torch.full((n, ld + offset), float("nan")).to(dtype)
    zt = (3.0 * torch.randn(n, v, generator=g)).to(dtype)
    zi = (zt.float() + 0.05 * torch.randn(n, v, generator=g)).to(dtype)
    store_t[:, offset:offset + v] = zt
    store_i[:, offset:offset + v] = zi
    ids = torch.randint(0, v, (n,), generator=g)
    ids[0] = 0
    ids[-1] = v - 1
    gout = torch.randn(n, generator=g)
    wl = workloads.RowWorkload(
        name="rand", z_train=store_t.to(device)[:, offset:offset + v],
        z_infer=store_i.to(device)[:, offset:offset + v], ids=ids.to(device),
        grad_out=gout.to(device), rhos=[])
    return wl


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("v", [1, 2, 7, 8, 16, 33, 1000, 2047, 4104, 8200, 20001, 33000, 70003])
def test_shapes_resident_path(dvp, dtype, v, gradient_steps):
    n = 5 if v > 20000 else 9
    es = 2 if dtype == torch.bfloat16 else 4
    ld = (v * es + 15) // 16 * 16 // es          # 16-byte aligned rows -> single-read kernel
    wl = _random_case(n, v, dtype, seed=v, ld=ld)
    code = 1 if dtype == torch.bfloat16 else 0
    p = dvp.DvpParams(n, v, ld, ld, ld, code, -1.0, code)
    # rows shorter than one 16-byte vector go to the streaming kernel
    assert dvp.lib().dvp_row_path(p, 1) == (1 if v * es >= 16 else 0)
    for rho in (1e-2, 0.0):
        _run_case(dvp, wl, rho, backward=True, threads=2)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("slots", [256 * 4, 256 * 8, 256 * 16, 1024 * 8, 1024 * 12, 1024 * 16, 1024 * 19, 1024 * 20])
@pytest.mark.parametrize("extra", ["one", "all_but_one"])
def test_membership_bits_when_whole_vectors_fill_every_register_slot(dvp, dtype, slots, extra):
    """Rows whose whole 16-byte vectors fill every slot of a kernel build exactly, plus a ragged end:
    the ragged end's bits have no slot of their own there.  The bit buffers start as all ones, so a word
    the kernel does not write shows."""
    epv = 8 if dtype == torch.bfloat16 else 4
    v = slots * epv + (1 if extra == "one" else epv - 1)
    n = 3
    ld = (v + epv - 1) // epv * epv
    wl = _random_case(n, v, dtype, seed=slots + len(extra), ld=ld)
    with torch.no_grad():       # ragged-end tokens on both sides of the threshold
        wl.z_train[0, v - 1] = 30.0
        wl.z_infer[1, v - 1] = 30.0
    for rho in (1e-2, 0.0):
        lr = dvp.log_rho(rho)
        out_t = dvp.SideOutputs(n, v, "cuda", lse_full=True, safe_bits=True)
        out_i = dvp.SideOutputs(n, v, "cuda", lse_full=True, safe_bits=True)
        out_t.safe_bits.fill_(-1)
        out_i.safe_bits.fill_(-1)
        res = dvp.dvp_forward(wl.z_train, wl.z_infer, wl.ids, lr, out_train=out_t, out_infer=out_i)
        torch.cuda.synchronize()
        ids = wl.ids.cpu()
        tol = parity.TOL[dtype]
        parity.check_side("train", res.train, wl.z_train.cpu(), ids, lr, tol, v, threads=4)
        parity.check_side("infer", res.infer, wl.z_infer.cpu(), ids, lr, tol, v, threads=4)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("v", [1, 5, 64, 1001, 5000, 40000])
def test_shapes_streaming_path_misaligned(dvp, dtype, v):
    # odd leading dimension and an element offset: rows are not 16-byte aligned
    wl = _random_case(6, v, dtype, seed=1000 + v, ld=v + 3, offset=1)
    assert wl.z_train.data_ptr() % 16 != 0
    for rho in (1e-2, 0.0):
        _run_case(dvp, wl, rho, backward=True, threads=2)


@pytest.mark.parametrize("dtype,v,ld", [
    (torch.bfloat16, 8 * 1024 * 20 + 8, None),        # one vector more than the registers hold
    (torch.bfloat16, 8 * 1024 * 20 + 8 * 1024 + 3, 8 * 1024 * 21 + 8),   # one more per thread, ragged end
    (torch.bfloat16, 262144, None),                   # a 256k vocabulary: 192 KB of every row outside the registers
    (torch.float32, 4 * 1024 * 20 + 4, None),
    (torch.float32, 151936, None),                    # fp32 logits at the 152k vocabulary
    (torch.float32, 100003, 100004)])
def test_rows_longer_than_the_register_file(dvp, dtype, v, ld, gradient_steps):
    """The first 1024 x 20 vectors of a row stay in registers, the rest is re-read in every phase by the
    same kernel: every output and both gradient forms (lists for short safe sets, dense rows) to the
    usual bars, membership bits included."""
    wl = _random_case(5, v, dtype, seed=v % 1000, ld=ld)
    code = 1 if dtype == torch.bfloat16 else 0
    p = dvp.DvpParams(5, v, ld or v, ld or v, ld or v, code, -1.0, code)
    assert dvp.lib().dvp_row_path(p, 1) == 1
    # put the sampled token of one row, and the row maximum of another, into the re-read part
    with torch.no_grad():
        wl.ids[1] = v - 5
        wl.z_train[2, v - 9] = 40.0
        wl.z_infer[2, v - 9] = 40.0
        wl.ids[2] = v - 9
    for rho in (1e-3, 1e-1, 0.0):       # dense rows, rows with a handful of safe tokens (lists), no pruning
        _run_case(dvp, wl, rho, backward=True, threads=4)
    _run_case(dvp, wl, 1e-2, backward=False, lse_full=False, bits=False, threads=4)


# ---------------------------------------------------------------------------
# degenerate rows
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_adversarial_rows(dvp, dtype, gradient_steps):
    v = 4104
    rows = []
    rows.append(torch.full((v,), -3.25))                       # all equal: every token safe
    r = torch.full((v,), -20.0); r[1234] = 7.5; rows.append(r)  # single spike
    r = torch.zeros(v); r[[0, v - 1, 77]] = 5.0; rows.append(r)  # ties at the maximum, first/last index
    r = torch.linspace(-30, 2, v); rows.append(r)               # a ramp crossing the threshold
    r = torch.randn(v); r[::3] = float("-inf"); rows.append(r)  # -inf entries
    r = torch.zeros(v); r[5] = 4.0; r[6] = 4.0 - 2.0; rows.append(r)   # token exactly at the threshold (log_rho = -2)
    r = 300.0 + torch.randn(v); rows.append(r)                  # large magnitudes
    r = -300.0 + torch.randn(v); rows.append(r)
    z = torch.stack(rows).to(dtype)
    n = z.shape[0]
    ids = torch.tensor([5, 1234, 77, v - 1, 1, 6, 10, 11])
    gout = torch.tensor([1.0, -1.0, 2.0, 0.5, -0.25, 1.0, 1.0, -3.0])
    zi = z.clone()
    zi[:, :16] = (zi[:, :16].float() * 1.01).to(dtype)
    wl = workloads.RowWorkload("adv", z.cuda(), zi.cuda(), ids.cuda(), gout.cuda(), [])
    tol = parity.TOL[dtype]
    for lr in (-2.0, float(parity.orc.log_rho_f32(1e-4)), 0.0, float("-inf")):
        res = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr,
                                       lse_full=True, safe_bits=True)
        torch.cuda.synchronize()
        # fp32 outputs carry half an ulp of |lse| (about 1.5e-5 at 300): widen the bound by it
        st = parity.check_side("train", res.train, z, ids, lr, max(tol, 4e-5), v, threads=2)
        si = parity.check_side("infer", res.infer, zi, ids, lr, max(tol, 4e-5), v, threads=2)
        parity.check_flags(res.row_flags, st["y_in_safe"], si["y_in_safe"], ids, v, train_safe_count=st["safe_count"])
        parity.check_gradient("dz", res.dz, z, ids, gout, lr, tol, threads=2)
        if lr == -2.0:
            assert st["safe_count"][0] == v and st["safe_count"][1] == 1 and st["safe_count"][2] == 3
            assert st["y_in_safe"][5] == 1        # boundary token is inside (Def. 5.1 uses >=)


def test_out_of_range_ids_are_flagged_not_faulted(dvp, gradient_steps):
    wl = _random_case(6, 1000, torch.bfloat16, seed=5)
    ids = wl.ids.clone()
    ids[1] = -1
    ids[2] = 1000
    ids[3] = 2 ** 40
    wl.ids = ids
    st = _run_case(dvp, wl, 1e-2, backward=True, threads=1)
    flags = st["result"].row_flags.cpu().numpy()
    assert list(flags[1:4] & 4) == [4, 4, 4] and (flags[0] & 4) == 0
    assert torch.all(st["result"].dz[1:4] == 0)


def test_empty_batch_and_no_infer_side(dvp):
    z = torch.empty(0, 128, dtype=torch.bfloat16, device="cuda")
    ids = torch.empty(0, dtype=torch.int64, device="cuda")
    g = torch.empty(0, device="cuda")
    res = dvp.dvp_forward_backward(z, z, ids, g, -3.0)
    assert res.dz.shape == (0, 128)
    wl = _random_case(7, 3000, torch.float32, seed=9)
    lr = dvp.log_rho(1e-3)
    res = dvp.dvp_forward(wl.z_train, None, wl.ids, lr, lse_full=True, safe_bits=True)
    torch.cuda.synchronize()
    st = parity.check_side("train", res.train, wl.z_train.cpu(), wl.ids.cpu(), lr, 1e-5, 3000)
    parity.check_flags(res.row_flags, st["y_in_safe"], None, wl.ids.cpu(), 3000, train_safe_count=st["safe_count"])


# ---------------------------------------------------------------------------
# split calls agree with the fused call; repeated runs are bit-identical
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_split_forward_then_backward_matches_oracle_and_fused(dvp, dtype):
    wl = _random_case(33, 12344, dtype, seed=21)
    lr = dvp.log_rho(1e-3)
    fwd = dvp.dvp_forward(wl.z_train, wl.z_infer, wl.ids, lr)
    dz = dvp.dvp_backward(wl.z_train, wl.ids, wl.grad_out, fwd.train.row_max, fwd.train.lse_safe,
                          fwd.row_flags, lr)
    fused = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr)
    torch.cuda.synchronize()
    parity.check_gradient("split dz", dz, wl.z_train.cpu(), wl.ids.cpu(), wl.grad_out.cpu(), lr,
                          parity.TOL[dtype], threads=4)
    assert torch.equal(fwd.train.logp, fused.train.logp)
    assert torch.equal(fwd.infer.logp, fused.infer.logp)
    assert torch.equal(fwd.row_flags, fused.row_flags)
    diff = (dz.float() - fused.dz.float()).abs().max().item()
    assert diff <= (1e-6 if dtype == torch.float32 else 2 ** -8 * 4)


def test_repeated_runs_are_bit_identical(dvp):
    wl = workloads.make_rows(1, device="cuda", n=300)
    lr = dvp.log_rho(1e-4)
    a = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, lse_full=True)
    b = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, lse_full=True)
    torch.cuda.synchronize()
    for k in ("logp", "row_max", "lse_safe", "lse_full", "safe_count"):
        assert torch.equal(getattr(a.train, k), getattr(b.train, k))
        assert torch.equal(getattr(a.infer, k), getattr(b.infer, k))
    assert torch.equal(a.dz.view(torch.int16), b.dz.view(torch.int16))


# ---------------------------------------------------------------------------
# full benchmark size, in the launch configuration the benchmark times:
# sampled rows against the oracle, plus properties that hold at any size
# ---------------------------------------------------------------------------
def _full_size_check(dvp, wl, rho, rows, bits_rows=256):
    """One fused call on the whole workload in the benchmark's launch configuration (lean build, caller's
    buffers), its outputs on `rows` (None: every row) against the oracle; then the membership bitmask and
    lse_full of a second call on the first `bits_rows` of those rows, bit by bit."""
    lr = dvp.log_rho(rho)
    n, v = wl.z_train.shape
    res = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr)
    torch.cuda.synchronize()
    rp = parity.compare_workload(wl, lr, res.train, res.infer, res.row_flags, res.dz, rows=rows, threads=16)
    out = rp.result()
    assert out["ok"], out
    sel = np.arange(n)[:bits_rows] if rows is None else rows[:bits_rows]
    idx = torch.as_tensor(sel, device="cuda")
    sub = workloads.RowWorkload("sub", wl.z_train[idx].contiguous(), wl.z_infer[idx].contiguous(),
                                wl.ids[idx].contiguous(), wl.grad_out[idx].contiguous(), [])
    ext = dvp.dvp_forward(sub.z_train, sub.z_infer, sub.ids, lr, lse_full=True, safe_bits=True)
    torch.cuda.synchronize()
    bits = parity.compare_workload(sub, lr, ext.train, ext.infer, ext.row_flags, None, threads=16,
                                   bits=(ext.train, ext.infer)).result()
    assert bits["ok"] and bits["membership_rows_checked"] == 2 * len(sel), bits
    print("rho %g: %d rows, logp err %.2e, gradient at %.3f of its bound (raw %.2e), %d rows with the sampled token "
          "pruned, %d tokens within 1e-6 of the ideal threshold" %
          (rho, out["rows_checked"], out["logp_max_abs_err"], out["grad_worst_ratio_to_bound"],
           out["grad_raw_max_abs_err"], out["rows_sampled_token_pruned_train"],
           out["band_tokens_train"] + out["band_tokens_infer"]))
    return out, res


@pytest.fixture
def default_gradient_steps(dvp):
    # the full-size tests run the configuration the benchmark times: the size decides how the gradient is written
    old = dvp.set_split_min_bytes(dvp.SPLIT_MIN_BYTES_DEFAULT)
    yield
    dvp.set_split_min_bytes(old)


def test_config1_full_size_every_row(dvp, default_gradient_steps):
    wl = workloads.make_rows(1, device="cuda")            # 2048 x 32000 bf16, thousands of safe tokens per row
    out, _ = _full_size_check(dvp, wl, 1e-4, None)        # (a 131 MB gradient: written by the row kernel alone)
    assert out["rows_checked"] == 2048


def test_config2_full_size_one_row_in_eight(dvp, default_gradient_steps):
    wl = workloads.make_rows(2, device="cuda")            # 8192 x 151936 bf16
    n, v = wl.z_train.shape
    rows = np.arange(0, n, 8)                             # 1024 rows; every fifth of them has a forced (uniform) token
    forced = wl.forced_rows.cpu().numpy()[rows]
    assert forced.sum() >= 50
    for rho in (1e-4, math.exp(-13.0), 0.0):
        out, res = _full_size_check(dvp, wl, rho, rows)
        assert out["rows_checked"] == 1024
        # any-size properties on every row
        cnt = res.train.safe_count
        assert int(cnt.min()) >= 1 and int(cnt.max()) <= v
        assert torch.all(res.train.lse_safe >= res.train.row_max)
        ys = (res.row_flags & 1).bool()
        assert torch.all(res.dz[~ys] == 0)
        assert torch.all(torch.isneginf(res.train.logp[~ys]))
        assert torch.all(res.train.logp[ys] <= 0)
        if rho == 0.0:
            assert torch.all(cnt == v)
        else:
            assert out["rows_sampled_token_pruned_train"] >= forced.sum() - 2
    del wl
    torch.cuda.empty_cache()


def _every_row_properties(wl, res, lr, chunk=1024):
    """What holds on every row whatever the size (Def. 5.1 / 5.2, Prop. 5.4), from the call's own outputs with torch
    on the GPU (no oracle): the safe set recounted from tau = fl32(m + log_rho) has the reported size, the pruned
    probabilities exp(z - lse_safe) over it sum to one, the gradient is zero outside it and sums to
    g (1 - sum of the pruned probabilities) ~ 0 over the row, and its entry at the sampled token is g (1 - p_y)."""
    n, v = wl.z_train.shape
    lr32 = torch.tensor(lr, dtype=torch.float32, device="cuda")
    worst = dict(prob_sum=0.0, grad_sum=0.0, grad_y=0.0)
    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        z = wl.z_train[r0:r1].float()
        m = res.train.row_max[r0:r1]
        assert torch.equal(m, z.max(dim=1).values)
        tau = (m + lr32).unsqueeze(1)                                        # one fp32 add, as in the kernel
        safe = z >= tau
        assert torch.equal(safe.sum(dim=1).to(torch.int32), res.train.safe_count[r0:r1])
        p = torch.where(safe, torch.exp(z.double() - res.train.lse_safe[r0:r1].double().unsqueeze(1)), torch.zeros((), dtype=torch.float64, device="cuda"))
        # lse_safe is an fp32 number near the row maximum (hundreds here): exp(z - lse_safe) carries its half unit
        lse_ulp = res.train.lse_safe[r0:r1].double().abs() * 2.0 ** -23 + 1e-6
        worst["prob_sum"] = max(worst["prob_sum"], ((p.sum(dim=1) - 1.0).abs() / lse_ulp).max().item())
        dz = res.dz[r0:r1].double()
        ys = (res.row_flags[r0:r1] & 1).bool()
        assert torch.count_nonzero(dz[~safe]).item() == 0                    # zero outside the safe set
        assert torch.count_nonzero(dz[~ys]).item() == 0                      # and on rows whose sampled token is pruned
        g = wl.grad_out[r0:r1].double()
        scale = g.abs().clamp(min=1.0)
        worst["grad_sum"] = max(worst["grad_sum"], (dz.sum(dim=1).abs() / scale)[ys].max().item())
        y = wl.ids[r0:r1]
        py = p.gather(1, y.unsqueeze(1)).squeeze(1)
        dzy = dz.gather(1, y.unsqueeze(1)).squeeze(1)
        worst["grad_y"] = max(worst["grad_y"], ((dzy - g * (1.0 - py)).abs() / scale)[ys].max().item())
        del z, safe, p, dz
    return worst


def test_config3_full_size_properties_on_every_row(dvp, default_gradient_steps):
    """Every one of the 32768 rows of the workload the headline figure is quoted on, at the headline threshold and
    with nothing pruned: the any-size properties above (bf16 gradient entries are rounded to 8 bits, so a row's
    gradient sums to zero within the roundings of its few large entries)."""
    wl = workloads.make_rows(3, device="cuda")
    for rho in (1e-4, 0.0):
        lr = dvp.log_rho(rho)
        res = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr)
        torch.cuda.synchronize()
        w = _every_row_properties(wl, res, lr)
        print("rho %g: |sum p - 1| <= %.2f units of lse_safe, |sum dz| / max(1,|g|) <= %.2e, |dz_y - g (1 - p_y)| / max(1,|g|) <= %.2e"
              % (rho, w["prob_sum"], w["grad_sum"], w["grad_y"]))
        assert w["prob_sum"] <= 1.0                # within one unit in the last place of the fp32 lse_safe
        assert w["grad_sum"] <= 2.0 ** -6          # the roundings of the row's few entries of magnitude up to |g| (2^-8 each)
        assert w["grad_y"] <= 2.0 ** -8 + 1e-6     # one bf16 rounding (half a unit of 8 bits) of an entry of magnitude at most |g|
        del res
    del wl
    torch.cuda.empty_cache()


def test_config3_full_size_every_threshold(dvp, default_gradient_steps):
    """The workload the headline figure is quoted on (32768 x 151936 bf16), at each of its four thresholds:
    2048 rows of the full-size call against the oracle, and nested safe sets across the thresholds."""
    wl = workloads.make_rows(3, device="cuda")
    n, v = wl.z_train.shape
    rows = np.arange(0, n, 16)
    counts = {}
    for rho in (1e-2, 1e-4, 1e-6, 0.0):
        out, res = _full_size_check(dvp, wl, rho, rows)
        assert out["rows_checked"] == 2048
        counts[rho] = res.train.safe_count.clone()
        del res
    assert torch.all(counts[1e-2] <= counts[1e-4]) and torch.all(counts[1e-4] <= counts[1e-6])   # Def. 5.1: nested in rho
    assert torch.all(counts[0.0] == v)
    del wl
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_rows_on_both_sides_of_the_list_capacity(dvp, dtype, gradient_steps):
    """Gaussian logits whose safe sets straddle the 64-token list capacity: some rows leave a list
    for the fill kernels, the others are written densely by the row kernel, in one call."""
    n, v = 48, 40000
    g = torch.Generator(device="cpu").manual_seed(4242)
    zt = (12.0 * torch.randn(n, v, generator=g)).to(dtype)
    zi = (zt.float() + 0.01 * torch.randn(n, v, generator=g)).to(dtype)
    ids = torch.argmax(zi.float(), dim=1)
    ids[5] = int(torch.argmin(zt[5].float()))            # a pruned sampled token among them
    wl = workloads.RowWorkload(name="gauss", z_train=zt.cuda(), z_infer=zi.cuda(), ids=ids.cuda(),
                               grad_out=torch.randn(n, generator=g).cuda(), rhos=[])
    res = dvp.dvp_forward(wl.z_train, wl.z_infer, wl.ids, dvp.log_rho(1e-6))
    torch.cuda.synchronize()
    counts = res.train.safe_count.cpu().numpy()
    assert (counts <= 64).sum() >= 5 and (counts > 64).sum() >= 5 and counts.max() < 2000
    _run_case(dvp, wl, 1e-6, backward=True, threads=4)


def test_a_million_short_rows(dvp):
    """Many more rows than workgroups, a row of three 16-byte vectors: every row against the oracle."""
    n, v = (1 << 20) + 3, 24
    g = torch.Generator(device="cuda").manual_seed(12)
    zt = (3.0 * torch.randn(n, v, generator=g, device="cuda")).to(torch.bfloat16)
    zi = (zt.float() + 0.05 * torch.randn(n, v, generator=g, device="cuda")).to(torch.bfloat16)
    ids = torch.randint(0, v, (n,), generator=g, device="cuda")
    go = torch.randn(n, generator=g, device="cuda")
    wl = workloads.RowWorkload(name="short", z_train=zt, z_infer=zi, ids=ids, grad_out=go, rhos=[])
    st = _run_case(dvp, wl, 1e-1, backward=True, threads=8)
    assert 0.05 < st["train"]["y_in_safe"].mean() < 0.95      # both kinds of rows in numbers
