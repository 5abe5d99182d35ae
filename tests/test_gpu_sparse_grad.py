"""GPU parity of dvp_forward_backward_sparse (gradient as per-row lists) against the fp64 oracle.

Bars: the index set of every row equals the oracle's safe set exactly (both
decide membership by the same fp32 threshold); grad_len, flags and all forward
outputs are bit-exact where integer; the values are fp32 and are held to the
fp32 gradient bound 1e-5 * max(1, |grad_out_i|) whatever the logits' storage
type (nothing is rounded to bf16 on this path); the per-row forward outputs
are identical to dvp_forward_backward's.
"""
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


def _check_lists(dvp, wl, rho, cap, rows=None):
    lr = dvp.log_rho(rho)
    res = dvp.dvp_forward_backward_sparse(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, cap)
    torch.cuda.synchronize()
    n, v = wl.z_train.shape
    sel = np.arange(n) if rows is None else np.asarray(rows)
    zt = wl.z_train[torch.as_tensor(sel, device=wl.z_train.device)].cpu()
    ids = wl.ids.cpu().numpy()[sel]
    g = wl.grad_out.cpu().numpy().astype(np.float64)[sel]
    o = orc.rows(zt, ids, np.float32(lr), grad_out=g, want_dz=True, want_flags=True, threads=8)
    flags = res.row_flags.cpu().numpy()[sel]
    glen = res.grad_len.cpu().numpy()[sel]
    want_len = np.where(o["y_in_safe"] == 1, o["safe_count"], 0)
    np.testing.assert_array_equal(glen, want_len)
    over = (want_len > cap)
    np.testing.assert_array_equal((flags & 8) != 0, over)
    np.testing.assert_array_equal(flags & 1, o["y_in_safe"])
    worst = 0.0
    for r, i in enumerate(sel):
        got = res.row(int(i))
        if over[r]:
            assert got is None
            continue
        idx, val = got
        want_idx = np.nonzero(o["safe_flags"][r])[0] if o["y_in_safe"][r] else np.zeros(0, np.int64)
        np.testing.assert_array_equal(idx.numpy(), want_idx, err_msg="row %d: index set" % i)
        if len(want_idx):
            err = np.abs(val.double().numpy() - o["dz"][r, want_idx]).max() / (1e-5 * max(1.0, abs(g[r])))
            worst = max(worst, err)
    assert worst <= 1.0, "list values off by %.2f x the fp32 bound" % worst
    return res, o, over


def test_small_safe_sets_large_vocab(dvp):
    # configs[2] shape, fewer rows: heavy tails, safe sets of a few tokens, 5 % pruned samples
    wl = workloads.make_rows(2, device="cuda", n=512)
    res, o, over = _check_lists(dvp, wl, 1e-4, 64)
    assert not over.any() and (o["y_in_safe"] == 0).sum() > 5
    # same forward outputs as the dense entry point, bit for bit
    lr = dvp.log_rho(1e-4)
    ref = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr)
    torch.cuda.synchronize()
    for side in ("train", "infer"):
        for k in ("logp", "row_max", "lse_safe", "safe_count"):
            assert torch.equal(getattr(getattr(res, side), k), getattr(getattr(ref, side), k)), (side, k)
    assert torch.equal(res.row_flags & 0xF7, ref.row_flags)          # all but the list-overflow bit
    # and the lists scatter to the dense gradient (bf16-rounded there)
    dense = ref.dz.float().cpu()
    for i in (0, 1, 20, 300):
        idx, val = res.row(i)
        row = torch.zeros(dense.shape[1])
        row[idx] = val
        assert torch.equal(row.bfloat16().float(), dense[i])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_thousands_of_safe_tokens_and_overflow(dvp, dtype):
    # configs[0]/[1] shape: safe sets of thousands; a capacity in the middle of their range overflows some rows
    wl = workloads.make_rows(0 if dtype == torch.float32 else 1, device="cuda", n=96, v=32000)
    if wl.grad_out is None:
        wl.grad_out = torch.randn(96, device="cuda")
    res, o, over = _check_lists(dvp, wl, 1e-4, 4000)
    assert over.any() and not over.all()
    _check_lists(dvp, wl, 1e-4, 65536)
    _check_lists(dvp, wl, 0.0, 32000)          # nothing pruned: every token listed


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("v", [9, 1000, 20011, 70003, 170003])
def test_ragged_vocab(dvp, dtype, v):
    # padded 16-byte aligned rows with a ragged end, sampled ids at both ends of the row
    from tests.test_gpu_rows import _random_case
    es = 2 if dtype == torch.bfloat16 else 4
    ld = (v * es + 15) // 16 * 16 // es
    wl = _random_case(7, v, dtype, seed=77 + v, ld=ld)
    cap = min(v, 65536)
    _check_lists(dvp, wl, 1e-2, cap)
    _check_lists(dvp, wl, 0.0, cap)            # from v = 70003 on every row overflows the largest list
    # (v = 170003: longer than the register file holds, the end of the row is re-read)
    _check_lists(dvp, wl, 1e-2, 3)


def test_argument_errors(dvp):
    wl = workloads.make_rows(1, device="cuda", n=8, v=20016)
    lr = dvp.log_rho(1e-3)
    with pytest.raises(dvp.DvpError) as e:
        dvp.dvp_forward_backward_sparse(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, 0)
    assert e.value.status == 3
    with pytest.raises(dvp.DvpError) as e:          # rows start on odd 2-byte boundaries: no single-read path
        z = wl.z_train.reshape(-1)[1:1 + 7 * 20016].reshape(7, 20016)
        dvp.dvp_forward_backward_sparse(z, None, wl.ids[:7], wl.grad_out[:7], lr, 64)
    assert e.value.status == 5


def test_full_size_sampled_rows(dvp):
    """configs[3] at full size (32768 x 151936 bf16), sampled rows against the oracle."""
    wl = workloads.make_rows(3, device="cuda")
    rng = np.random.default_rng(3)
    n = wl.z_train.shape[0]
    rows = np.unique(np.concatenate([[0, n - 1], rng.choice(n, 62, replace=False), np.arange(0, 200, 20)]))
    _check_lists(dvp, wl, 1e-4, 256, rows=rows)
    del wl
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# dense gradient from the saved lists (grad_out known only after the forward)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_lists_to_dense_matches_the_fused_gradient(dvp, dtype):
    """Forward with grad_out = 1 and lists, then dz = grad_out * lists: the dense matrix equals the
    oracle's to the usual gradient bar; rows whose list overflowed are taken from the logits."""
    n, v = 40, 40000
    g = torch.Generator().manual_seed(99)
    zt = (12.0 * torch.randn(n, v, generator=g)).to(dtype)              # safe sets from a handful to hundreds
    zi = (zt.float() + 0.01 * torch.randn(n, v, generator=g)).to(dtype)
    ids = torch.argmax(zi.float(), dim=1)
    ids[3] = int(torch.argmin(zt[3].float()))                           # a pruned sampled token: zero row
    go = torch.randn(n, generator=g)
    zt, zi, ids, go = zt.cuda(), zi.cuda(), ids.cuda(), go.cuda()
    lr = dvp.log_rho(1e-6)
    ones = torch.ones(n, device="cuda")
    cap = 64
    sp = dvp.dvp_forward_backward_sparse(zt, zi, ids, ones, lr, cap)
    torch.cuda.synchronize()
    over = (sp.row_flags.cpu().numpy() & 8) != 0
    assert 3 < over.sum() < n - 3                                        # both kinds of rows are present
    dz = torch.full((n, v), 7.0, dtype=dtype, device="cuda")             # stale contents must not survive
    dvp.dvp_lists_to_dense(sp, v, dtype, go, lr, z_train=zt, ids=ids, dz=dz)
    torch.cuda.synchronize()
    tol = parity.TOL[dtype]
    parity.check_gradient("dz from lists", dz, zt.cpu(), ids.cpu(), go.cpu(), lr, tol, threads=4)
    # without the logits the overflowing rows are left alone, the others are identical
    dz2 = torch.full((n, v), 7.0, dtype=dtype, device="cuda")
    dvp.dvp_lists_to_dense(sp, v, dtype, go, lr, dz=dz2)
    torch.cuda.synchronize()
    keep = torch.as_tensor(~over, device="cuda")
    assert torch.equal(dz2[keep], dz[keep])
    assert torch.all(dz2[~keep] == 7.0)
    # no scale: the lists as they are
    dz3 = dvp.dvp_lists_to_dense(sp, v, dtype, None, lr)
    torch.cuda.synchronize()
    idx, val = sp.row(int(np.nonzero(~over)[0][0]))
    row = dz3[int(np.nonzero(~over)[0][0])].float().cpu()
    assert torch.equal(row[idx], val.to(dtype).float()) and row.abs().sum() == val.to(dtype).float().abs().sum()


def test_lists_to_dense_ragged_and_padded(dvp):
    from tests.test_gpu_rows import _random_case
    v, ld = 20011, 20016
    wl = _random_case(7, v, torch.bfloat16, seed=5, ld=ld)
    lr = dvp.log_rho(1e-2)
    sp = dvp.dvp_forward_backward_sparse(wl.z_train, wl.z_infer, wl.ids, torch.ones(7, device="cuda"), lr, 4096)
    store = torch.full((7, ld + 3), 7.0, dtype=torch.bfloat16, device="cuda")
    for dz in (store[:, :v], store[:, 1:v + 1]):                       # 16-byte aligned rows, then odd ones
        store.fill_(7.0)
        dvp.dvp_lists_to_dense(sp, v, torch.bfloat16, wl.grad_out, lr, dz=dz)
        torch.cuda.synchronize()
        parity.check_gradient("dz", dz, wl.z_train.cpu(), wl.ids.cpu(), wl.grad_out.cpu(), lr, 2e-3, threads=2)
    assert torch.all(store[:, v + 1:] == 7.0) and torch.all(store[:, 0] == 7.0)   # nothing outside the rows
