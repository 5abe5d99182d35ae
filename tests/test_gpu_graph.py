"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
memset nodes), so a call sequence can be captured in a HIP graph and replayed.  Each replay is compared
bit for bit with the same calls made eagerly on the same inputs, with the inputs changed and eager work
done between the replays."""
import numpy as np
import pytest
import torch

from paper_2512_23087_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dvp():
    from paper_2512_23087_amd import dvp as binding
    binding.lib()
    return binding


def _row_buffers(dvp, n, v, like):
    return dict(out_train=dvp.SideOutputs(n, v, "cuda"), out_infer=dvp.SideOutputs(n, v, "cuda"),
                row_flags=torch.empty(n, dtype=torch.uint8, device="cuda"), dz=torch.empty_like(like))


def test_rows_and_sequence_step_replayed_from_a_graph(dvp):
    n, v = 96, 40000
    wl = workloads.make_rows(2, device="cuda", n=n, v=v)
    other = workloads.make_rows(3, device="cuda", n=n, v=v)
    lr, lthr = dvp.log_rho(1e-4), dvp.log_threshold(1e-4)
    off = torch.tensor([0, 10, 10, 57, 96], dtype=torch.int64, device="cuda")
    zt, zi = wl.z_train.clone(), wl.z_infer.clone()
    ids, go = wl.ids.clone(), wl.grad_out.clone()

    def run(bufs, seq):
        dvp.dvp_forward_backward(zt, zi, ids, go, lr, **bufs)
        dvp.dvp_sequence_weights(bufs["out_train"].logp, bufs["out_infer"].logp, off, lthr, **seq)

    def seq_buffers():
        return dict(weight=torch.empty(n, device="cuda"), seq_log_ratio=torch.empty(4, device="cuda"),
                    seq_min_weight=torch.empty(4, device="cuda"), seq_veto=torch.empty(4, dtype=torch.uint8, device="cuda"))

    eager, eager_seq = _row_buffers(dvp, n, v, zt), seq_buffers()
    graph_b, graph_seq = _row_buffers(dvp, n, v, zt), seq_buffers()
    run(eager, eager_seq)                       # warm-up: one-time occupancy queries happen outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(graph_b, graph_seq)
    for rep in range(4):
        if rep == 1:                            # new logits, ids and upstream gradients in the captured buffers
            zt.copy_(other.z_train); zi.copy_(other.z_infer); ids.copy_(other.ids); go.copy_(other.grad_out)
        if rep == 2:
            zt.copy_(wl.z_train); ids.copy_(wl.ids)
        if rep == 3:
            graph_b["dz"].fill_(7.0)            # stale output contents must not matter
        run(eager, eager_seq)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(graph_b["dz"], eager["dz"]), rep
        assert torch.equal(graph_b["row_flags"], eager["row_flags"])
        for side in ("out_train", "out_infer"):
            for k in ("logp", "row_max", "lse_safe", "safe_count"):
                a, b = getattr(graph_b[side], k), getattr(eager[side], k)
                assert torch.equal(torch.nan_to_num(a.float(), nan=-1.0), torch.nan_to_num(b.float(), nan=-1.0)), (rep, side, k)
        for k in graph_seq:
            assert torch.equal(torch.nan_to_num(graph_seq[k].float(), nan=-1.0),
                               torch.nan_to_num(eager_seq[k].float(), nan=-1.0)), (rep, k)
    assert graph_b["dz"].float().abs().max().item() > 0


def test_lmhead_replayed_from_a_graph(dvp):
    wl = workloads.make_lmhead(device="cuda", n=300, d=128, v=1500)
    wl2 = workloads.make_lmhead(device="cuda", n=300, d=128, v=1500)
    lr = dvp.log_rho(1e-4)
    hidden = wl.hidden.clone()
    ws = torch.empty(dvp.lmhead_workspace_bytes(300, 128, 1500), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty_like(ws)
    dh, dw = torch.empty(300, 128, device="cuda"), torch.empty(1500, 128, device="cuda")
    dh2, dw2 = torch.empty_like(dh), torch.empty_like(dw)
    # the binding allocates the per-row output arrays itself: keep the first call's and capture that call
    first = dvp.dvp_fused_lmhead(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, workspace=ws2, d_hidden=dh2, d_w=dw2)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        res = dvp.dvp_fused_lmhead(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, workspace=ws, d_hidden=dh, d_w=dw)
    for rep in range(3):
        if rep == 1:
            hidden.copy_((wl2.hidden.float() * 1.5).to(torch.bfloat16))
        ref = dvp.dvp_fused_lmhead(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, workspace=ws2, d_hidden=dh2, d_w=dw2)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(dh, dh2) and torch.equal(dw, dw2), rep
        assert torch.equal(res.train.logp, ref.train.logp) and torch.equal(res.infer.logp, ref.infer.logp)
        assert torch.equal(res.row_flags, ref.row_flags)
    assert first.train.logp.shape == res.train.logp.shape


def test_lmhead_list_form_replayed_from_a_graph(dvp):
    """The list form decides on the device which rows need a second pass: one captured graph serves
    inputs that need none and inputs with flat rows among the peaked ones."""
    n, d, v, cap = 300, 128, 3000, 64
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v, hidden_scale=60.0)
    lr = dvp.log_rho(1e-4)
    hidden = wl.hidden.clone()
    flat = wl.hidden.clone()
    flat[::29] = (flat[::29].float() * 1e-3).to(torch.bfloat16)
    import ctypes
    p = dvp.DvpLmHeadParams(n, d, v, d, d, lr)
    nbytes = int(dvp.lib().dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(p), cap))
    ws, ws2 = (torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(2))
    bufs = [dict(d_hidden=torch.empty(n, d, device="cuda"), d_w=torch.empty(v, d, device="cuda"),
                 entries=torch.zeros(n, cap, 2, dtype=torch.int32, device="cuda"),
                 grad_len=torch.empty(n, dtype=torch.int32, device="cuda")) for _ in range(2)]
    dvp.dvp_fused_lmhead_lists(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, cap, workspace=ws2, **bufs[1])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        res = dvp.dvp_fused_lmhead_lists(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, cap, workspace=ws, **bufs[0])
    want_second = [0, len(range(0, n, 29)), 0]
    for rep in range(3):
        hidden.copy_(flat if rep == 1 else wl.hidden)
        ref = dvp.dvp_fused_lmhead_lists(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, cap, workspace=ws2, **bufs[1])
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert res.second_pass.tolist() == [want_second[rep]] * 2 == ref.second_pass.tolist(), rep
        assert torch.equal(bufs[0]["d_hidden"], bufs[1]["d_hidden"]) and torch.equal(bufs[0]["d_w"], bufs[1]["d_w"]), rep
        assert torch.equal(res.grad_len, ref.grad_len) and torch.equal(res.row_flags, ref.row_flags)
        valid = torch.arange(cap, device="cuda")[None, :] < torch.where((res.row_flags & 8) != 0, 0, res.grad_len)[:, None]
        assert torch.equal(bufs[0]["entries"][valid], bufs[1]["entries"][valid])
        for side in ("train", "infer"):
            for k in ("logp", "row_max", "lse_safe", "safe_count"):
                assert torch.equal(getattr(getattr(res, side), k), getattr(getattr(ref, side), k)), (rep, side, k)


def test_lists_and_counted_dense_rows_replayed_from_a_graph(dvp):
    """The list form followed by the dense gradient of its flagged rows, chosen and counted on the device: one
    captured graph serves inputs with no flagged row, with some, and with others, and matches eager calls."""
    n, d, v, cap, max_rows = 300, 128, 3000, 64, 80
    wl = workloads.make_lmhead(device="cuda", n=n, d=d, v=v, hidden_scale=60.0)
    lr = dvp.log_rho(1e-4)
    import ctypes
    p = dvp.DvpLmHeadParams(n, d, v, d, d, lr)
    nbytes = int(dvp.lib().dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(p), cap))
    rbytes = int(dvp.lib().dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(p), max_rows))
    hidden = wl.hidden.clone()
    variants = [wl.hidden.clone() for _ in range(3)]
    variants[1][::29] = (variants[1][::29].float() * 0.05).to(torch.bfloat16)
    variants[2][5::17] = (variants[2][5::17].float() * 0.05).to(torch.bfloat16)

    def buffers():
        return dict(ws=torch.empty(nbytes, dtype=torch.uint8, device="cuda"), wr=torch.empty(rbytes, dtype=torch.uint8, device="cuda"),
                    d_hidden=torch.empty(n, d, device="cuda"), d_w=torch.empty(v, d, device="cuda"),
                    entries=torch.zeros(n, cap, 2, dtype=torch.int32, device="cuda"),
                    grad_len=torch.empty(n, dtype=torch.int32, device="cuda"),
                    rows=torch.empty(max_rows, dtype=torch.int32, device="cuda"),
                    n_sub=torch.empty(1, dtype=torch.int32, device="cuda"))

    def run(b):
        res = dvp.dvp_fused_lmhead_lists(hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr, cap, workspace=b["ws"],
                                         d_hidden=b["d_hidden"], d_w=b["d_w"], entries=b["entries"], grad_len=b["grad_len"])
        dvp.dvp_fused_lmhead_select_rows(res.row_flags, dvp.ROW_GRAD_OVERFLOW, b["rows"], b["n_sub"])
        dvp.dvp_fused_lmhead_rows_counted(hidden, wl.w_train, wl.ids, wl.grad_out, lr, b["rows"], b["n_sub"], b["d_hidden"],
                                          b["d_w"], workspace=b["wr"])
        return res

    eager, graph = buffers(), buffers()
    run(eager)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        res_g = run(graph)
    counts = []
    for rep in (0, 1, 2, 0):
        hidden.copy_(variants[rep])
        res_e = run(eager)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        counts.append(int(graph["n_sub"].item()))
        assert graph["n_sub"].item() == eager["n_sub"].item() == int(((res_e.row_flags & 8) != 0).sum().item())
        assert torch.equal(graph["d_hidden"], eager["d_hidden"]) and torch.equal(graph["d_w"], eager["d_w"]), rep
        assert torch.equal(res_g.row_flags, res_e.row_flags)
    assert counts[0] == 0 and counts[1] > 5 and counts[2] > 5 and counts[1] != counts[2] and counts[3] == 0


def test_concurrent_callers_on_their_own_streams(dvp):
    """The library keeps no state between calls: host threads with a stream each get the same results
    as one thread."""
    import threading
    wls = [workloads.make_rows(2, device="cuda", n=64, v=40000), workloads.make_rows(3, device="cuda", n=64, v=32000)]
    lr = dvp.log_rho(1e-4)
    ref = [dvp.dvp_forward_backward(w.z_train, w.z_infer, w.ids, w.grad_out, lr) for w in wls]
    torch.cuda.synchronize()
    out, errs = [None, None], []

    def work(i):
        try:
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.default_stream())
            with torch.cuda.stream(s):
                for _ in range(20):
                    out[i] = dvp.dvp_forward_backward(wls[i].z_train, wls[i].z_infer, wls[i].ids, wls[i].grad_out, lr)
            s.synchronize()
        except Exception as e:          # noqa: BLE001 - reported below
            errs.append(e)

    ts = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    assert not errs, errs
    for i in range(2):
        assert torch.equal(out[i].dz, ref[i].dz) and torch.equal(out[i].train.logp, ref[i].train.logp)
        assert torch.equal(out[i].row_flags, ref[i].row_flags)


FRESH_PROCESS = r"""
import sys
import torch
from paper_2512_23087_amd import dvp, workloads

dvp.prepare()                               # the only library call before the capture
wl = workloads.make_rows(2, device="cuda", n=64, v=40000)
lm = workloads.make_lmhead(device="cuda", n=300, d=128, v=1500)
lr = dvp.log_rho(1e-4)
ws = torch.empty(dvp.lmhead_workspace_bytes(300, 128, 1500), dtype=torch.uint8, device="cuda")
dh, dw = torch.empty(300, 128, device="cuda"), torch.empty(1500, 128, device="cuda")
torch.cuda.synchronize()
g = torch.cuda.CUDAGraph()
with torch.cuda.graph(g):
    rows = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, lse_full=True, safe_bits=True)
    head = dvp.dvp_fused_lmhead(lm.hidden, lm.w_train, lm.w_infer, lm.ids, lm.grad_out, lr, workspace=ws,
                                d_hidden=dh, d_w=dw)
for rep in range(2):
    g.replay()
    torch.cuda.synchronize()
    ref = dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, lr, lse_full=True, safe_bits=True)
    ref_head = dvp.dvp_fused_lmhead(lm.hidden, lm.w_train, lm.w_infer, lm.ids, lm.grad_out, lr)
    torch.cuda.synchronize()
    assert torch.equal(rows.dz, ref.dz) and torch.equal(rows.train.logp, ref.train.logp), rep
    assert torch.equal(rows.train.safe_bits, ref.train.safe_bits) and torch.equal(rows.row_flags, ref.row_flags), rep
    assert torch.equal(dh, ref_head.d_hidden) and torch.equal(dw, ref_head.d_w), rep
    assert torch.equal(head.train.logp, ref_head.train.logp) and torch.equal(head.infer.logp, ref_head.infer.logp), rep
print("fresh-process capture ok")
"""


def test_capture_as_the_first_call_of_a_fresh_process_after_prepare():
    """dvp_prepare() does every kernel build's one-time host set-up (occupancy queries, LDS limits), so the
    very first call of an entry point can already sit inside a stream capture.  Runs in a process of its
    own: in this one earlier tests have made those first calls."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", FRESH_PROCESS], cwd=root, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0 and "fresh-process capture ok" in res.stdout, res.stdout[-2000:] + res.stderr[-4000:]
