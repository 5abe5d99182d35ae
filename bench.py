#!/usr/bin/env python3
"""Benchmark of the DVP row path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2] [--rho 1e-4]

One step = one dvp_forward_backward call over the whole batch: both logit
matrices are read, every per-row output and the full gradient matrix are
written.  Inputs are generated on the GPU beforehand and are resident in HBM
when the timed region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the
# same counters' reading on a plain copy kernel of known size.  Only valid for the kernel
# source it was measured on: keyed by the sha256 of the kernel sources.
MEASURED_TRAFFIC = {
    # sha256 of csrc/dvp_rows.hip + dvp_device.h + dvp_internal.h -> HBM bytes per launch; see
    # profiles/rows_cfg3_hbm_traffic.md for the counter values and scale factors
    "da5f035eb7ab63057ccd3c378112de220225eed736ba3fc25b28182308f7454c": {"cfg3": 29894924000},
}


def kernel_source_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in ("dvp_rows.hip", "dvp_device.h", "dvp_internal.h"):
        with open(os.path.join(ROOT, "paper_2512_23087_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def algorithmic_bytes_per_row(vocab: int, elem: int, infer_elem: int) -> int:
    """What the method must move per row: read the training row, read the
    inference row, write the gradient row, plus the per-row scalars
    (id 8, grad_out 4, and per side logp/row_max/lse_safe/safe_count 16; flags 1)."""
    return 2 * vocab * elem + vocab * infer_elem + 8 + 4 + 16 * 2 + 1


def cpu_baseline(wl, log_rho, target_seconds=12.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import dvp_oracle as orc
    threads = min(os.cpu_count() or 1, 16)
    n = wl.z_train.shape[0]

    chunk = 512
    done, spent, r0 = 0, 0.0, 0
    while spent < target_seconds:            # walks the workload's rows, wrapping around if it is short
        r1 = min(n, r0 + chunk)
        zt = wl.z_train[r0:r1].cpu()
        zi = wl.z_infer[r0:r1].cpu()
        ids = wl.ids[r0:r1].cpu().numpy()
        g = wl.grad_out[r0:r1].cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        orc.rows(zt, ids, np.float32(log_rho), grad_out=g, want_dz=True, threads=threads)
        orc.rows(zi, ids, np.float32(log_rho), threads=threads)
        spent += time.perf_counter() - t0
        done += r1 - r0
        r0 = r1 if r1 < n else 0
    return {"value": done / spent, "unit": "rows/s", "cores": threads, "kind": "oracle",
            "sample": "%d rows of the workload in chunks of %d (wrapping around after its %d rows), forward "
                      "(both sides) + backward, fp64 C oracle on %d threads, %.1f s of CPU wall time"
                      % (done, chunk, n, threads, spent)}


def time_launches(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        starts[i].record()
        fn()
        ends[i].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_launch_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    return wall, per_launch_ms


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix peak
MFMA_FP8_PEAK_TFLOPS = 5000.0    # and dense fp8


def bench_lmhead(args):
    """configs[4]: the LM-head variant (logits never stored).  One step = one
    dvp_fused_lmhead call: both sides' forward and the training side's dH, dW."""
    import torch
    from paper_2512_23087_amd import dvp, workloads
    f8 = args.infer_dtype == "f8"
    wl = workloads.make_lmhead(device="cuda:0", n=args.rows, f8_engine=f8, hidden_scale=args.hidden_scale,
                               flat_every=args.flat_every)
    lists_cap = args.sparse_grad            # --sparse-grad on this workload: the gradient kept as per-row lists
    if lists_cap and args.split_lists:
        print("bench.py: --sparse-grad on the lmhead workload does not go with --split-lists", file=sys.stderr)
        sys.exit(2)
    n, d = wl.hidden.shape
    v = wl.w_train.shape[0]
    lr = dvp.log_rho(args.rho)
    if lists_cap:
        import ctypes
        pl = dvp.DvpLmHeadParams(n, d, v, wl.hidden.stride(0), wl.w_train.stride(0), lr)
        ws = torch.empty(int(dvp.lib().dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(pl), lists_cap)),
                         dtype=torch.uint8, device="cuda:0")
        entries = torch.empty(n, lists_cap, 2, dtype=torch.int32, device="cuda:0")
        grad_len = torch.empty(n, dtype=torch.int32, device="cuda:0")
    else:
        ws = torch.empty(dvp.lmhead_workspace_bytes(n, d, v), dtype=torch.uint8, device="cuda:0")
    dh = torch.empty(n, d, dtype=torch.float32, device="cuda:0")
    dw = torch.empty(v, d, dtype=torch.float32, device="cuda:0")

    two_calls = bool(args.split_lists)      # --split-lists on this workload: forward and backward as two calls
    if two_calls:
        p = dvp.DvpLmHeadParams(n, d, v, wl.hidden.stride(0), wl.w_train.stride(0), lr)
        import ctypes
        saved = torch.empty(int(dvp.lib().dvp_fused_lmhead_saved_bytes(ctypes.byref(p))), dtype=torch.uint8,
                            device="cuda:0")

    last = {}
    over_rows = ws_rows = None
    if lists_cap and args.dense_rows:
        # the rows over the list cap, found once (the inputs do not change between steps; a training loop
        # reads row_flags back each step or keeps an upper bound), and the workspace of their dense call
        first = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, wl.grad_out, lr,
                                           lists_cap, workspace=ws, d_hidden=dh, d_w=dw, entries=entries, grad_len=grad_len,
                                           infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None)
        over_rows = torch.nonzero((first.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).squeeze(1).to(torch.int32)
        ws_rows = torch.empty(max(int(dvp.lib().dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(pl), over_rows.numel())), 256),
                              dtype=torch.uint8, device="cuda:0")

    def step():
        if lists_cap:
            last["res"] = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, wl.grad_out, lr,
                                                     lists_cap, workspace=ws, d_hidden=dh, d_w=dw, entries=entries,
                                                     grad_len=grad_len,
                                                     infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None)
            if over_rows is not None and over_rows.numel():
                dvp.dvp_fused_lmhead_rows(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, over_rows, dh, dw, workspace=ws_rows)
        elif two_calls:
            _, kept = dvp.dvp_fused_lmhead_forward(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, lr,
                                                   infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None,
                                                   saved=saved, workspace=ws)
            dvp.dvp_fused_lmhead_backward(kept, wl.grad_out, d_hidden=dh, d_w=dw)
        elif f8:
            dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, workspace=ws, d_hidden=dh,
                                 d_w=dw, infer_f8=(wl.hidden8, wl.w8, wl.scale_infer))
        else:
            dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr,
                                 workspace=ws, d_hidden=dh, d_w=dw)

    steps = min(args.steps, 5)
    wall, per_launch = time_launches(step, steps, min(args.warmup, 2))
    ms = sum(per_launch) / len(per_launch)
    gemm = 2.0 * n * v * d
    useful, executed = 4 * gemm, 6 * gemm          # train fwd, infer fwd, dH, dW; vs the passes actually run
    extra = {}
    if lists_cap:
        res = last["res"]
        over = int(((res.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).sum().item())
        listed = int(torch.where((res.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0, torch.zeros_like(res.grad_len),
                                 res.grad_len).sum().item())
        # two forwards as matrix products (one pass each, two where a side needed its second pass), the
        # gradient as |lists| x d multiply-adds, twice
        second = [int(x) for x in res.second_pass.cpu().tolist()]      # rows of each side that went through a second pass
        passes = 2 + sum(second) / n
        useful, executed = 2 * gemm + 4.0 * listed * d, passes * gemm + 4.0 * listed * d
        n_f8_passes = (1 + second[1] / n) if f8 else 0.0
        if over_rows is not None:       # the dense call on those rows: its two forward passes and the two gradient products
            dense = 4.0 * over_rows.numel() / n
            passes += dense
            executed += dense * gemm
            useful += 2.0 * over_rows.numel() / n * gemm
            extra_dense = {"dense_rows": int(over_rows.numel())}
        extra = {"list_cap": lists_cap, "list_entries": listed, "rows_over_cap": over, "gemm_passes": passes, "second_pass_rows": second,
                 "mean_safe_set": float(res.train.safe_count.float().mean().item())}
        if over_rows is not None:
            extra.update(extra_dense)
            extra["gemm_passes"] = passes
    # (each side's forward produces the logits twice: row max first, then sums at the threshold)
    # Peak for the mix of passes: each contraction is priced at the peak of its own operand type, so the
    # call's floor is sum(flop_i / peak_i) and the peak quoted is executed flop over that floor.
    n_f8 = (n_f8_passes if lists_cap else 2) if f8 else 0
    floor_s = ((executed / gemm - n_f8) * gemm / MFMA_BF16_PEAK_TFLOPS + n_f8 * gemm / MFMA_FP8_PEAK_TFLOPS) / 1e12
    peak = executed / floor_s / 1e12
    result = {
        "metric": "DVP fused LM-head fwd+bwd rows/s and MFMA TFLOP/s, V=%d bf16" % v,
        "value": n * steps / wall, "unit": "rows/s", "n_gpus": 1, "steps": steps,
        "warmup": min(args.warmup, 2), "ms_per_step": wall * 1e3 / steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16+f8" if f8 else "bf16", "data": "synthetic",
        "config": {"workload": ("configs[4]: hidden [%d, %d] bf16 x W [%d, %d] bf16 (train); inference side an 8-bit "
                                "engine: E4M3 activations and head with per-tensor factors, rho=%g" if f8 else
                                "configs[4]: hidden [%d, %d] bf16 x W [%d, %d] bf16 (train) and its "
                                "fp8-e4m3-rounded copy (infer), rho=%g") % (n, d, v, d, args.rho)
                               + (", hidden states scaled by %g (peaked rows)" % args.hidden_scale
                                  if args.hidden_scale != 1.0 else "")
                               + (", every %d-th row left at scale 1 (flat)" % args.flat_every if args.flat_every else ""),
                   "entry_point": (("dvp_fused_lmhead_lists_f8infer" if f8 else "dvp_fused_lmhead_lists")
                                   + (" + dvp_fused_lmhead_rows" if over_rows is not None else "")) if lists_cap else
                                  "dvp_fused_lmhead_forward + dvp_fused_lmhead_backward" if two_calls else
                                  "dvp_fused_lmhead_f8infer" if f8 else "dvp_fused_lmhead",
                   "workspace_bytes": ws.numel(), "saved_bytes": saved.numel() if two_calls else 0, **extra},
        "roofline": {"bound": "mfma", "achieved": executed / (ms * 1e-3) / 1e12,
                     "peak": peak, "unit": "TFLOP/s",
                     "frac": executed / (ms * 1e-3) / 1e12 / peak, "traffic": None,
                     "kernel": "gemm_nt_kernel (%.4g GEMM passes of 2*N*V*d flop each per call%s)"
                               % (extra.get("gemm_passes", 6), ": 4 bf16 at 2.5 PFLOP/s peak, 2 fp8 at 5.0" if f8 else ""),
                     "kernel_ms_avg": ms, "executed_tflop": executed / 1e12,
                     "useful_tflop": useful / 1e12,
                     "useful_tflops": useful / (ms * 1e-3) / 1e12},
    }
    print(json.dumps(result))


def bench_sequences(args):
    """Sequence-level step (importance weights, cumulative mismatch, token veto) on the paper's batch
    shape (Sec. 6): 32 sampled sequences of up to 16384 tokens.  One step = one dvp_sequence_weights call."""
    import numpy as np
    import torch
    from paper_2512_23087_amd import dvp
    g = torch.Generator(device="cuda:0"); g.manual_seed(0xD5B0 + 5)
    lens = torch.randint(8192, 16385, (32,), generator=g, device="cuda:0")
    off = torch.cat([torch.zeros(1, dtype=torch.int64, device="cuda:0"), torch.cumsum(lens, 0)])
    n = int(off[-1].item())
    lt = -3.0 * torch.rand(n, generator=g, device="cuda:0")
    li = lt + 0.02 * torch.randn(n, generator=g, device="cuda:0")
    lthr = dvp.log_threshold(1e-4)
    w = torch.empty(n, dtype=torch.float32, device="cuda:0")
    r = torch.empty(32, dtype=torch.float32, device="cuda:0")
    mn = torch.empty(32, dtype=torch.float32, device="cuda:0")
    veto = torch.empty(32, dtype=torch.uint8, device="cuda:0")

    def step():
        dvp.dvp_sequence_weights(lt, li, off, lthr, weight=w, seq_log_ratio=r, seq_min_weight=mn, seq_veto=veto)

    wall, per_launch = time_launches(step, args.steps, args.warmup)
    ms = sum(per_launch) / len(per_launch)
    nbytes = 12 * n + 33 * 8 + 32 * 9          # two fp32 log-probs in, one weight out per token; offsets; per-sequence outputs
    result = {
        "metric": "DVP sequence weights tokens/s and achieved HBM GB/s", "value": n * args.steps / wall,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "32 sequences of 8192..16384 tokens (%d tokens), veto threshold 1e-4" % n,
                   "entry_point": "dvp_sequence_weights"},
        "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "sequence_kernel (32 workgroups: launch-latency bound at this size)",
                     "kernel_ms_avg": ms, "algorithmic_bytes_per_launch": nbytes},
    }
    if not args.no_cpu_baseline:
        from oracle import dvp_oracle as orc
        a, b, o = lt.cpu().numpy(), li.cpu().numpy(), off.cpu().numpy()
        t0 = time.perf_counter(); reps = 0
        while time.perf_counter() - t0 < 10.0:
            orc.sequences(a, b, o, np.float32(lthr)); reps += 1
        spent = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n * reps / spent, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                  "sample": "%d passes of the fp64 C oracle over the same %d tokens, %.1f s" % (reps, n, spent)}
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "lmhead", "seq"])
    ap.add_argument("--rho", type=float, default=1e-4)
    ap.add_argument("--rows", type=int, default=None, help="override N (for quick runs)")
    ap.add_argument("--sparse-grad", type=int, default=0, metavar="CAP",
                    help="deliver the gradient as per-row (index, value) lists of at most CAP entries "
                         "(dvp_forward_backward_sparse) instead of the dense matrix")
    ap.add_argument("--split-lists", type=int, default=0, metavar="CAP",
                    help="(with --workload lmhead, any CAP > 0: one step = dvp_fused_lmhead_forward + "
                         "dvp_fused_lmhead_backward)  "
                         "the flow of a caller that learns grad_out only after the forward: one step = "
                         "dvp_forward_backward_sparse with grad_out = 1 (lists of at most CAP entries) followed by "
                         "dvp_lists_to_dense with the real grad_out (dense gradient, logits not read again)")
    ap.add_argument("--hidden-scale", type=float, default=1.0,
                    help="(lmhead workload) multiply the hidden states: 20 gives peaked rows with a few safe tokens "
                         "each; with --sparse-grad CAP one step = dvp_fused_lmhead_lists")
    ap.add_argument("--dense-rows", action="store_true",
                    help="(lmhead workload with --sparse-grad) one step = the list-form call followed by "
                         "dvp_fused_lmhead_rows on the rows over the list cap: the gradient of every row")
    ap.add_argument("--flat-every", type=int, default=0, metavar="K",
                    help="(lmhead workload, with --hidden-scale) every K-th row keeps the scale 1: flat rows among peaked ones")
    ap.add_argument("--infer-dtype", default="same", choices=["same", "f8"],
                    help="f8: the inference logits are rounded through E4M3 (saturating) and handed over as "
                         "one byte per token")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run 3 plain device-to-device copies of one logits matrix (known "
                         "size: reads and writes N*V*elem bytes each) to calibrate HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; rows are independent, so N GPUs would each "
              "take N_rows/N rows with no communication. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_23087_amd import dvp, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the DVP library has no CPU path", file=sys.stderr)
        sys.exit(2)
    dvp.lib()
    torch.cuda.set_device(0)
    if args.workload == "lmhead":
        return bench_lmhead(args)
    if args.workload == "seq":
        return bench_sequences(args)
    cfg = int(args.workload[-1])
    t_gen = time.perf_counter()
    wl = workloads.make_rows(cfg, device="cuda:0", n=args.rows)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    n, v = wl.z_train.shape
    elem = wl.z_train.element_size()
    lr = dvp.log_rho(args.rho)
    if args.infer_dtype == "f8":
        zi8 = torch.empty(n, v, dtype=torch.float8_e4m3fn, device="cuda:0")
        for r0 in range(0, n, 1024):
            zi8[r0:r0 + 1024] = workloads.through_e4m3(wl.z_infer[r0:r0 + 1024].float()).to(torch.float8_e4m3fn)
        wl.z_infer = zi8
        torch.cuda.synchronize()
    infer_elem = wl.z_infer.element_size()

    out_t = dvp.SideOutputs(n, v, wl.z_train.device)
    out_i = dvp.SideOutputs(n, v, wl.z_train.device)
    flags = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    dz = torch.empty_like(wl.z_train)

    if args.split_lists:
        cap = args.split_lists
        entries = torch.empty(n, cap, 2, dtype=torch.int32, device="cuda:0")
        glen = torch.empty(n, dtype=torch.int32, device="cuda:0")
        ones = torch.ones(n, dtype=torch.float32, device="cuda:0")

        def step(log_rho_value=lr):
            sp = dvp.dvp_forward_backward_sparse(wl.z_train, wl.z_infer, wl.ids, ones, log_rho_value, cap,
                                                 out_train=out_t, out_infer=out_i, row_flags=flags,
                                                 entries=entries, grad_len=glen)
            dvp.dvp_lists_to_dense(sp, v, wl.z_train.dtype, wl.grad_out, log_rho_value, z_train=wl.z_train,
                                   ids=wl.ids, dz=dz)
    elif args.sparse_grad:
        del dz
        entries = torch.empty(n, args.sparse_grad, 2, dtype=torch.int32, device="cuda:0")
        glen = torch.empty(n, dtype=torch.int32, device="cuda:0")

        def step(log_rho_value=lr):
            dvp.dvp_forward_backward_sparse(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, log_rho_value,
                                            args.sparse_grad, out_train=out_t, out_infer=out_i,
                                            row_flags=flags, entries=entries, grad_len=glen)
    else:
        def step(log_rho_value=lr):
            dvp.dvp_forward_backward(wl.z_train, wl.z_infer, wl.ids, wl.grad_out, log_rho_value,
                                     out_train=out_t, out_infer=out_i, row_flags=flags, dz=dz)

    if args.copy_probe:
        for _ in range(3):
            dz.copy_(wl.z_train)
        torch.cuda.synchronize()
    wall, per_launch = time_launches(step, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = sum(per_launch) / len(per_launch)
    bytes_per_launch = algorithmic_bytes_per_row(v, elem, infer_elem) * n
    if args.sparse_grad:
        # no dense gradient row; the lists that were written (8 bytes per entry) and their lengths instead
        listed = glen[(flags & 8) == 0].to(torch.int64).sum().item()
        bytes_per_launch += -v * elem * n + 8 * listed + 4 * n
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9

    traffic = MEASURED_TRAFFIC.get(kernel_source_hash(), {}).get(args.workload) \
        if args.rows is None and args.rho == 1e-4 and not args.sparse_grad and not args.split_lists \
        and args.infer_dtype == "same" else None

    result = {
        "metric": "DVP fwd+bwd rows/s and achieved HBM GB/s (% of peak), V=151936 bf16",
        "value": n * args.steps / wall,
        "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[%d]: N=%d x V=%d %s logits (train + infer%s), fused "
                               "forward+backward, rho=%g" % (cfg, n, v, str(wl.z_train.dtype)[6:],
                                                             ", inference logits as E4M3 bytes" if infer_elem == 1 else "",
                                                             args.rho),
                   "storage_dtype": str(wl.z_train.dtype)[6:], "infer_storage_dtype": str(wl.z_infer.dtype)[6:],
                   "n_rows": n, "vocab": v,
                   "rho": args.rho,
                   "entry_point": "dvp_forward_backward_sparse (grad_out = 1, list capacity %d) + dvp_lists_to_dense"
                                  % args.split_lists if args.split_lists else
                                  "dvp_forward_backward_sparse (list capacity %d)" % args.sparse_grad
                                  if args.sparse_grad else "dvp_forward_backward",
                   "row_kernel": "resident" if dvp.lib().dvp_row_path(
                       dvp.DvpParams(n, v, v, v, v, 1 if elem == 2 else 0, lr,
                                     2 if infer_elem == 1 else (1 if elem == 2 else 0)), 1) == 1 else "streaming",
                   "input_generation_s": round(t_gen, 2)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "rows_resident_kernel (lists) + lists_zero_kernel + lists_scatter_kernel (+ "
                               "backward_kernel on overflowing rows); durations summed" if args.split_lists else
                               "rows_resident_kernel (gradient as lists)" if args.sparse_grad else
                               "rows_resident_kernel + grad_zero_kernel + grad_scatter_kernel "
                               "(one dvp_forward_backward call; durations summed)",
                     "kernel_ms_avg": kernel_ms, "kernel_ms_min": min(per_launch),
                     "algorithmic_bytes_per_launch": bytes_per_launch},
    }

    # safe-set sizes at the headline threshold, and the threshold sweep of configs[3]
    cnt = out_t.safe_count.to(torch.float64)
    result["safe_set"] = {"mean": cnt.mean().item(), "median": cnt.median().item(),
                          "max": cnt.max().item(),
                          "y_in_train_safe_frac": (flags & 1).to(torch.float64).mean().item()}
    if args.sparse_grad:
        result["overflow_rows"] = int(((flags & 8) != 0).sum().item())
    if args.split_lists:
        result["overflow_rows"] = int(((flags & 8) != 0).sum().item())
        # the lists are written once and read once on top of the dense figure
        listed = glen[(flags & 8) == 0].to(torch.int64).sum().item()
        result["roofline"]["list_bytes_per_launch"] = 16 * listed
    if not args.no_sweep and not args.sparse_grad:
        sweep = []
        for rho in wl.rhos:
            lr_s = dvp.log_rho(rho)
            w, pl = time_launches(lambda: step(lr_s), max(3, args.steps // 3), 2)
            k_ms = sum(pl) / len(pl)
            c = out_t.safe_count
            edges = [1, 2, 4, 16, 256, 4096, 65536, v + 1]
            hist = torch.bucketize(c.to(torch.int64), torch.tensor(edges, device=c.device), right=True)
            sweep.append({"rho": rho, "kernel_ms_avg": k_ms,
                          "rows_per_s": n / (k_ms * 1e-3),
                          "hbm_frac": bytes_per_launch / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "safe_size_hist": {"edges": edges,
                                             "counts": torch.bincount(hist, minlength=len(edges) + 1).tolist()}})
        result["threshold_sweep"] = sweep

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, lr)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
