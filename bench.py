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

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the same
# counters' reading on a plain copy kernel of known size.  A figure is only valid for the kernel
# sources it was measured on: the table is keyed by the sha256 of those sources, then by the run's
# configuration; see profiles/rows_*_hbm_traffic.md for the counter values and scale factors.
# A run whose sources or configuration have no entry reports "traffic": null, "traffic_stale": true.
MEASURED_TRAFFIC = {
    "71b5ffbd96474e94f6ed13f9ab79d80cb73cdb4b66dfa98240e54f23f30e6117": {
        "cfg3/rho=0.0001": 29902097257,                     # profiles/rows_cfg3_hbm_traffic.md
        "cfg3/rho=0": 29888018094,                          # profiles/rows_cfg3_rho0_hbm_traffic.md
        "cfg2/rho=0.0001": 7476724585,                      # profiles/rows_cfg2_hbm_traffic.md
        "cfg1/rho=0.0001": 394668532,                       # profiles/rows_cfg1_hbm_traffic.md
        "cfg3/rho=0.0001/lists=64": 19929263163,            # profiles/rows_cfg3_lists_hbm_traffic.md
        "cfg3/rho=0.0001/entry=backward": 19429795740,      # profiles/rows_cfg3_backward_hbm_traffic.md
    },
}


def kernel_source_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in ("dvp_rows.hip", "dvp_device.h", "dvp_internal.h", "dvp_api.hip"):
        with open(os.path.join(ROOT, "paper_2512_23087_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def traffic_key(args) -> str:
    """Names the configuration a traffic figure belongs to."""
    key = "%s/rho=%g" % (args.workload, args.rho)
    if args.entry != "fused":
        key += "/entry=" + args.entry
    if args.rows is not None:
        key += "/rows=%d" % args.rows
    if args.sparse_grad:
        key += "/lists=%d" % args.sparse_grad
    if args.split_lists:
        key += "/split=%d" % args.split_lists
    if args.infer_dtype != "same":
        key += "/infer=" + args.infer_dtype
    return key


def algorithmic_bytes_per_row(vocab: int, elem: int, infer_elem: int) -> int:
    """What the method must move per row: read the training row, read the
    inference row, write the gradient row, plus the per-row scalars
    (id 8, grad_out 4, and per side logp/row_max/lse_safe/safe_count 16; flags 1)."""
    return 2 * vocab * elem + vocab * infer_elem + 8 + 4 + 16 * 2 + 1


def host_threads() -> int:
    return min(os.cpu_count() or 1, 16)


def oracle_one_core(wl, log_rho, rows=1024):
    """The fp64 oracle on ONE thread over the first rows of the workload: rows/s."""
    import numpy as np
    from oracle import dvp_oracle as orc
    n = min(rows, wl.z_train.shape[0])
    spent = 0.0
    for r0 in range(0, n, 256):
        r1 = min(n, r0 + 256)
        zt, zi = wl.z_train[r0:r1].cpu(), wl.z_infer[r0:r1].cpu()
        ids = wl.ids[r0:r1].cpu().numpy()
        g = wl.grad_out[r0:r1].cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        orc.rows(zt, ids, np.float32(log_rho), grad_out=g, want_dz=True, threads=1)
        orc.rows(zi, ids, np.float32(log_rho), threads=1)
        spent += time.perf_counter() - t0
    return n / spent, n, spent


def time_launches(fn, steps, warmup):
    """W untimed calls, then K calls between two synchronisations: wall time of the K calls and each
    call's duration from HIP events recorded around it on the stream it is launched on."""
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


def median(xs):
    ys = sorted(xs)
    k = len(ys)
    return ys[k // 2] if k % 2 else 0.5 * (ys[k // 2 - 1] + ys[k // 2])


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix peak
MFMA_FP8_PEAK_TFLOPS = 5000.0    # and dense fp8
EXECUTED_TRAIN_PASSES, EXECUTED_INFER_PASSES = 3, 1   # GEMM passes dvp_fused_lmhead runs per side (forward + dH + dW; forward)


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
        # The rows over the list cap get their dense gradient from a second call.  Which rows those are, and
        # how many, stays on the device (dvp_fused_lmhead_select_rows / dvp_fused_lmhead_rows_counted): the
        # host only provides an upper bound, taken here from one look before the timed region (a training
        # loop would keep a bound of its own) and rounded up to a whole row tile.
        first = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, wl.grad_out, lr,
                                           lists_cap, workspace=ws, d_hidden=dh, d_w=dw, entries=entries, grad_len=grad_len,
                                           infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None)
        over_rows = torch.nonzero((first.row_flags & dvp.ROW_GRAD_OVERFLOW) != 0).squeeze(1).to(torch.int32)
        max_rows = max(256, -(-over_rows.numel() // 256) * 256)
        rows_buf = torch.empty(max_rows, dtype=torch.int32, device="cuda:0")
        n_sub_dev = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        ws_rows = torch.empty(max(int(dvp.lib().dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(pl), max_rows)), 256),
                              dtype=torch.uint8, device="cuda:0")

    def step():
        if lists_cap:
            last["res"] = dvp.dvp_fused_lmhead_lists(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, wl.grad_out, lr,
                                                     lists_cap, workspace=ws, d_hidden=dh, d_w=dw, entries=entries,
                                                     grad_len=grad_len,
                                                     infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None)
            if over_rows is not None:
                dvp.dvp_fused_lmhead_select_rows(last["res"].row_flags, dvp.ROW_GRAD_OVERFLOW, rows_buf, n_sub_dev)
                dvp.dvp_fused_lmhead_rows_counted(wl.hidden, wl.w_train, wl.ids, wl.grad_out, lr, rows_buf, n_sub_dev, dh, dw,
                                                  workspace=ws_rows)
        elif two_calls:
            fwd, kept = dvp.dvp_fused_lmhead_forward(wl.hidden, wl.w_train, None if f8 else wl.w_infer, wl.ids, lr,
                                                     infer_f8=(wl.hidden8, wl.w8, wl.scale_infer) if f8 else None,
                                                     saved=saved, workspace=ws)
            dvp.dvp_fused_lmhead_backward(kept, wl.grad_out, d_hidden=dh, d_w=dw)
            fwd.d_hidden, fwd.d_w = dh, dw
            last["res"] = fwd
        elif f8:
            last["res"] = dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, None, wl.ids, wl.grad_out, lr, workspace=ws,
                                               d_hidden=dh, d_w=dw, infer_f8=(wl.hidden8, wl.w8, wl.scale_infer))
        else:
            last["res"] = dvp.dvp_fused_lmhead(wl.hidden, wl.w_train, wl.w_infer, wl.ids, wl.grad_out, lr,
                                               workspace=ws, d_hidden=dh, d_w=dw)

    steps = min(args.steps, 5)
    wall, per_launch = time_launches(step, steps, min(args.warmup, 2))
    ms = sum(per_launch) / len(per_launch)
    gemm = 2.0 * n * v * d
    # useful: train forward, inference forward, dH, dW; executed: each side's forward produces the logits
    # twice (row maxima first, then the sums at the threshold)
    useful, executed = 4 * gemm, (EXECUTED_TRAIN_PASSES + EXECUTED_INFER_PASSES) * gemm
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
        if over_rows is not None:       # the dense call on those rows: its forward product and the two gradient products
            dense = 3.0 * over_rows.numel() / n
            passes += dense
            executed += dense * gemm
            useful += 2.0 * over_rows.numel() / n * gemm
            extra_dense = {"dense_rows": int(over_rows.numel())}
        extra = {"list_cap": lists_cap, "list_entries": listed, "rows_over_cap": over, "gemm_passes": passes, "second_pass_rows": second,
                 "mean_safe_set": float(res.train.safe_count.float().mean().item())}
        if over_rows is not None:
            extra.update(extra_dense)
            extra["gemm_passes"] = passes
    # Peak for a mix of passes: each contraction is priced at the peak of its own operand type, so a
    # call's floor is sum(flop_i / peak_i) and the peak quoted is its flop over that floor.  The roofline
    # fraction is on the USEFUL flop (the method's own work: train forward, inference forward, dH, dW,
    # or the list form's shorter sums); the passes actually executed are reported beside it.
    def mixed_peak(total_flop, f8_flop):
        return total_flop / ((total_flop - f8_flop) / MFMA_BF16_PEAK_TFLOPS + f8_flop / MFMA_FP8_PEAK_TFLOPS)
    n_f8 = (n_f8_passes if lists_cap else EXECUTED_INFER_PASSES) if f8 else 0
    peak_exec = mixed_peak(executed, n_f8 * gemm)
    peak_useful = mixed_peak(useful, gemm if f8 else 0.0)
    useful_rate = useful / (ms * 1e-3) / 1e12
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
                                   + (" + dvp_fused_lmhead_select_rows + dvp_fused_lmhead_rows_counted (no host read-back)"
                                      if over_rows is not None else "")) if lists_cap else
                                  "dvp_fused_lmhead_forward + dvp_fused_lmhead_backward" if two_calls else
                                  "dvp_fused_lmhead_f8infer" if f8 else "dvp_fused_lmhead",
                   "workspace_bytes": ws.numel(), "saved_bytes": saved.numel() if two_calls else 0, **extra},
        "roofline": {"bound": "mfma", "achieved": useful_rate, "peak": peak_useful, "unit": "TFLOP/s",
                     "frac": useful_rate / peak_useful, "traffic": None, "basis": "useful flop",
                     "kernel": "gemm_nt_kernel (%.4g GEMM passes of 2*N*V*d flop each executed per call%s)"
                               % (executed / gemm, "; bf16 passes priced at 2.5 PFLOP/s, fp8 passes at 5.0" if f8 else ""),
                     "kernel_ms_avg": ms, "kernel_ms_median": median(per_launch), "kernel_ms_min": min(per_launch),
                     "timed_launches": len(per_launch),
                     "useful_tflop": useful / 1e12, "executed_tflop": executed / 1e12,
                     "gemm_passes_executed": executed / gemm, "gemm_passes_useful": useful / gemm,
                     "executed_tflops": executed / (ms * 1e-3) / 1e12, "executed_peak": peak_exec,
                     "executed_frac": executed / (ms * 1e-3) / 1e12 / peak_exec},
    }
    # ---- sampled rows of the last timed call against the oracle (fp64 logits from the stored H and W with
    # ---- a BLAS matrix product, then the row oracle), and that oracle's speed as the CPU baseline
    if not args.no_cpu_baseline:
        import numpy as np
        from tests import parity
        torch.cuda.synchronize()
        rng = np.random.default_rng(4)
        k = min(n, args.parity_rows if args.parity_rows > 0 else 256)
        rows = np.unique(np.concatenate([[0, n - 1], rng.choice(n, k - 2, replace=False)])) if k > 2 else np.arange(k)
        threads = host_threads()
        res = last.get("res")
        if lists_cap:       # rows over the list cap carry no dH in the list form: forward outputs only
            import types
            res = types.SimpleNamespace(train=res.train, infer=res.infer, d_hidden=None)
        band = 2e-3 if f8 else 2e-4
        chk, spent = parity.lmhead_sampled_rows(wl, res, rows, lr, band=band, threads=threads,
                                                infer_scale=wl.scale_infer if f8 else None)
        chk.update(what="outputs of the last timed call on %d sampled token rows: forward of both sides%s" %
                        (len(rows), " and the rows of dH" if res.d_hidden is not None else ""), of_rows=n, rho=args.rho)
        result["parity"] = {"ok": chk["ok"], "checks": [chk]}
        from threadpoolctl import threadpool_limits
        one = rows[:8]
        with threadpool_limits(limits=1):
            _, spent1 = parity.lmhead_sampled_rows(wl, res, one, lr, band=band, threads=1,
                                                   infer_scale=wl.scale_infer if f8 else None)
        result["cpu_baseline"] = {
            "value": len(rows) / spent, "unit": "rows/s", "cores": threads, "kind": "oracle",
            "value_1core": len(one) / spent1,
            "sample": "fp64 oracle with BLAS matrix products for the logits (H W^T of both sides, and dz W for dH) and the "
                      "C row oracle on them: %d sampled rows on %d threads in %.1f s, %d rows on 1 thread in %.1f s; the "
                      "full workload is %d rows, so the whole-job figure is this rate as it stands (no dW in it)"
                      % (len(rows), threads, spent, len(one), spent1, n)}
    print(json.dumps(result))
    if result.get("parity") and not result["parity"]["ok"]:
        print("bench.py: the timed outputs do NOT match the oracle", file=sys.stderr)
        sys.exit(1)


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
    ap.add_argument("--steps", type=int, default=50)
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
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="leave the oracle out: no cpu_baseline, no parity check of the timed outputs")
    ap.add_argument("--parity-rows", type=int, default=0, metavar="K",
                    help="check about K evenly spaced rows of the timed call against the oracle instead of every row")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--entry", default="fused", choices=["fused", "split", "backward"],
                    help="row workloads: one step = dvp_forward_backward (fused, the default), dvp_forward followed by "
                         "dvp_backward (split), or dvp_backward alone on a forward done beforehand (backward)")
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
    return bench_rows(args)


def bench_rows(args):
    """configs[1..3]: one step = one fused forward+backward call over the whole batch."""
    import numpy as np
    import torch
    from paper_2512_23087_amd import dvp, workloads

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

    # Buffer sets.  A working set smaller than the 256 MB last-level cache would be served from it, so
    # such a workload (configs[1]: 393 MB per set, close to it) is rotated over several copies of its
    # inputs and outputs: every call then finds its rows in HBM, as a training step would.
    set_bytes = n * v * (2 * elem + infer_elem)
    n_sets = 1 if set_bytes > (2 << 30) else max(3, -(-(1 << 30) // set_bytes))
    sets = []
    for k in range(n_sets):
        sets.append(dict(
            zt=wl.z_train if k == 0 else wl.z_train.clone(), zi=wl.z_infer if k == 0 else wl.z_infer.clone(),
            ids=wl.ids if k == 0 else wl.ids.clone(), go=wl.grad_out if k == 0 else wl.grad_out.clone(),
            out_t=dvp.SideOutputs(n, v, wl.z_train.device), out_i=dvp.SideOutputs(n, v, wl.z_train.device),
            flags=torch.empty(n, dtype=torch.uint8, device="cuda:0"),
            dz=None if args.sparse_grad else torch.empty_like(wl.z_train)))
    cap = args.split_lists or args.sparse_grad
    if cap:
        for b in sets:
            b["entries"] = torch.empty(n, cap, 2, dtype=torch.int32, device="cuda:0")
            b["glen"] = torch.empty(n, dtype=torch.int32, device="cuda:0")
        ones = torch.ones(n, dtype=torch.float32, device="cuda:0")
    turn = [0]

    def step(log_rho_value=lr):
        b = sets[turn[0] % n_sets]
        turn[0] += 1
        if args.split_lists:
            sp = dvp.dvp_forward_backward_sparse(b["zt"], b["zi"], b["ids"], ones, log_rho_value, cap,
                                                 out_train=b["out_t"], out_infer=b["out_i"], row_flags=b["flags"],
                                                 entries=b["entries"], grad_len=b["glen"])
            dvp.dvp_lists_to_dense(sp, v, b["zt"].dtype, b["go"], log_rho_value, z_train=b["zt"], ids=b["ids"], dz=b["dz"])
        elif args.sparse_grad:
            dvp.dvp_forward_backward_sparse(b["zt"], b["zi"], b["ids"], b["go"], log_rho_value, cap,
                                            out_train=b["out_t"], out_infer=b["out_i"], row_flags=b["flags"],
                                            entries=b["entries"], grad_len=b["glen"])
        elif args.entry == "fused":
            dvp.dvp_forward_backward(b["zt"], b["zi"], b["ids"], b["go"], log_rho_value,
                                     out_train=b["out_t"], out_infer=b["out_i"], row_flags=b["flags"], dz=b["dz"])
        else:
            if args.entry == "split" or b.get("forward_at") != log_rho_value:
                dvp.dvp_forward(b["zt"], b["zi"], b["ids"], log_rho_value, out_train=b["out_t"], out_infer=b["out_i"],
                                row_flags=b["flags"])
                b["forward_at"] = log_rho_value
            dvp.dvp_backward(b["zt"], b["ids"], b["go"], b["out_t"].row_max, b["out_t"].lse_safe, b["flags"], log_rho_value,
                             dz=b["dz"])
        return b

    if args.copy_probe:
        for _ in range(3):
            sets[0]["dz"].copy_(wl.z_train)
        torch.cuda.synchronize()
    wall, per_launch = time_launches(step, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    kernel_ms = sum(per_launch) / len(per_launch)
    last = sets[(turn[0] - 1) % n_sets]                 # the buffer set the last timed call wrote
    out_t, out_i, flags, dz = last["out_t"], last["out_i"], last["flags"], last["dz"]
    bytes_per_launch = algorithmic_bytes_per_row(v, elem, infer_elem) * n
    if args.entry == "split":        # the training row is read a second time by the backward
        bytes_per_launch += v * elem * n
    if args.entry == "backward":     # training row in, gradient row out; id, grad_out, row_max, lse_safe, flags per row
        bytes_per_launch = (2 * v * elem + 8 + 4 + 4 + 4 + 1) * n
    if args.sparse_grad:
        # no dense gradient row; the lists that were written (8 bytes per entry) and their lengths instead
        listed = last["glen"][(flags & 8) == 0].to(torch.int64).sum().item()
        bytes_per_launch += -v * elem * n + 8 * listed + 4 * n
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9

    traffic = MEASURED_TRAFFIC.get(kernel_source_hash(), {}).get(traffic_key(args))

    dense_call = not args.sparse_grad and not args.split_lists and args.entry == "fused"
    # dvp_forward_backward finishes a large gradient with two write-only kernels (see dvp_set_split_min_bytes)
    two_steps = lr != float("-inf") and n * v * elem >= dvp.set_split_min_bytes(-1)
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
                   "buffer_sets": n_sets,
                   "entry_point": "dvp_forward_backward_sparse (grad_out = 1, list capacity %d) + dvp_lists_to_dense"
                                  % args.split_lists if args.split_lists else
                                  "dvp_forward_backward_sparse (list capacity %d)" % args.sparse_grad
                                  if args.sparse_grad else {"fused": "dvp_forward_backward", "split": "dvp_forward + dvp_backward",
                                                            "backward": "dvp_backward"}[args.entry],
                   "row_kernel": "resident" if dvp.lib().dvp_row_path(
                       dvp.DvpParams(n, v, v, v, v, 1 if elem == 2 else 0, lr,
                                     2 if infer_elem == 1 else (1 if elem == 2 else 0)), 1) == 1 else "streaming",
                   "input_generation_s": round(t_gen, 2)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_stale": traffic is None,
                     "kernel": "rows_resident_kernel (lists) + lists_zero_kernel + lists_scatter_kernel (+ "
                               "backward_kernel on overflowing rows); durations summed" if args.split_lists else
                               "rows_resident_kernel (gradient as lists)" if args.sparse_grad else
                               ("rows_resident_kernel + grad_zero_kernel + grad_scatter_kernel "
                                "(one dvp_forward_backward call; durations summed)" if two_steps else
                                "rows_resident_kernel (one dvp_forward_backward call; a gradient of this size, or with "
                                "nothing pruned, is written by the row kernel alone)") if args.entry == "fused" else
                               ("rows_resident_kernel (forward) + " if args.entry == "split" else "") +
                               "backward_zero_kernel + backward_kernel (durations summed)",
                     "kernel_ms_avg": kernel_ms, "kernel_ms_median": median(per_launch),
                     "kernel_ms_min": min(per_launch), "timed_launches": len(per_launch),
                     "frac_at_median": bytes_per_launch / (median(per_launch) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": bytes_per_launch},
    }

    # safe-set sizes at the headline threshold
    cnt = out_t.safe_count.to(torch.float64)
    result["safe_set"] = {"mean": cnt.mean().item(), "median": cnt.median().item(),
                          "max": cnt.max().item(),
                          "y_in_train_safe_frac": (flags & 1).to(torch.float64).mean().item()}
    if args.sparse_grad:
        result["overflow_rows"] = int(((flags & 8) != 0).sum().item())
    if args.split_lists:
        result["overflow_rows"] = int(((flags & 8) != 0).sum().item())
        # the lists are written once and read once on top of the dense figure
        listed = last["glen"][(flags & 8) == 0].to(torch.int64).sum().item()
        result["roofline"]["list_bytes_per_launch"] = 16 * listed

    # ---- parity of the timed call's outputs with the fp64 oracle (outside the timed region), and the
    # ---- oracle's own speed on the same rows as the CPU baseline
    use_oracle = not args.no_cpu_baseline
    threads = host_threads()
    sample = np.arange(0, n, max(1, n // 2048), dtype=np.int64)      # the rows checked at the sweep's other thresholds
    parity_out = None

    def membership_bits(b, log_rho_value):
        """An untimed dvp_forward with lse_full and the membership bitmask on a gathered copy of the
        sampled rows (the timed call runs the lean build), compared bit by bit with the oracle."""
        from tests import parity
        idx = torch.as_tensor(sample, device="cuda:0")
        sub = workloads.RowWorkload("sample", b["zt"][idx].contiguous(), b["zi"][idx].contiguous(),
                                    b["ids"][idx].contiguous(), b["go"][idx].contiguous(), [])
        res = dvp.dvp_forward(sub.z_train, sub.z_infer, sub.ids, log_rho_value, lse_full=True, safe_bits=True)
        torch.cuda.synchronize()
        return parity.compare_workload(sub, log_rho_value, res.train, res.infer, res.row_flags, None, threads=threads,
                                       bits=(res.train, res.infer)).result()

    def with_bits(chk, bits):
        chk["membership_bit_mismatches"] = bits["membership_bit_mismatches"]
        chk["membership_rows_checked"] = bits["membership_rows_checked"]
        chk["lse_full_max_abs_err"] = bits["lse_full_max_abs_err"]
        chk["ok"] = bool(chk["ok"] and bits["ok"])
        return chk

    if use_oracle and dense_call:
        from tests import parity
        torch.cuda.synchronize()
        view = workloads.RowWorkload("timed", last["zt"], last["zi"], last["ids"], last["go"], [])
        rows_all = None if args.parity_rows <= 0 or args.parity_rows >= n else \
            np.arange(0, n, max(1, n // args.parity_rows), dtype=np.int64)
        t0 = time.perf_counter()
        rp = parity.compare_workload(view, lr, out_t, out_i, flags, dz, rows=rows_all, threads=threads)
        head = rp.result()
        head["rho"] = args.rho
        head["of_rows"] = n
        head["what"] = "outputs of the last timed call, %s" % ("every row" if rows_all is None else "every %d-th row" % (n // args.parity_rows))
        with_bits(head, membership_bits(last, lr))
        head["seconds"] = round(time.perf_counter() - t0, 1)
        parity_out = {"ok": head["ok"], "checks": [head]}
        one_rate, one_rows, one_s = oracle_one_core(view, lr)
        result["cpu_baseline"] = {
            "value": rp.rows / rp.oracle_seconds, "unit": "rows/s", "cores": threads, "kind": "oracle",
            "value_1core": one_rate,
            "sample": "fp64 C oracle, forward (both sides) + backward: %d rows of the workload on %d threads in %.1f s "
                      "(the same pass that checks the timed outputs); %d rows on 1 thread in %.1f s"
                      % (rp.rows, threads, rp.oracle_seconds, one_rows, one_s)}

    if not args.no_sweep and not args.sparse_grad:
        sweep = []
        for rho in wl.rhos:
            lr_s = dvp.log_rho(rho)
            w, pl = time_launches(lambda: step(lr_s), max(3, args.steps // 3), 2)
            k_ms = sum(pl) / len(pl)
            b = sets[(turn[0] - 1) % n_sets]
            c = b["out_t"].safe_count
            edges = [1, 2, 4, 16, 256, 4096, 65536, v + 1]
            hist = torch.bucketize(c.to(torch.int64), torch.tensor(edges, device=c.device), right=True)
            sweep.append({"rho": rho, "kernel_ms_avg": k_ms, "kernel_ms_median": median(pl),
                          "rows_per_s": n / (k_ms * 1e-3),
                          "hbm_frac": bytes_per_launch / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                          "safe_size_hist": {"edges": edges,
                                             "counts": torch.bincount(hist, minlength=len(edges) + 1).tolist()}})
            if use_oracle and dense_call and rho != args.rho:
                from tests import parity
                view = workloads.RowWorkload("timed", b["zt"], b["zi"], b["ids"], b["go"], [])
                t0 = time.perf_counter()
                rp = parity.compare_workload(view, lr_s, b["out_t"], b["out_i"], b["flags"], b["dz"], rows=sample, threads=threads)
                chk = with_bits(rp.result(), membership_bits(b, lr_s))
                chk.update(rho=rho, of_rows=n, what="outputs of the last timed call at this threshold, %d rows (every %d-th)"
                           % (len(sample), max(1, n // 2048)), seconds=round(time.perf_counter() - t0, 1))
                parity_out["checks"].append(chk)
                parity_out["ok"] = bool(parity_out["ok"] and chk["ok"])
        result["threshold_sweep"] = sweep

    result["parity"] = parity_out

    # ---- what the machine delivers for this call's traffic mixes with no arithmetic at all (same buffers,
    # ---- same session): reads only, writes only, and rows read twice and written once from one workgroup
    if dense_call and not args.no_sweep and infer_elem == elem and v * elem <= 19 * 16384 and (v * elem) % 16 == 0:
        b = sets[0]

        def probe(mode):
            _, pl = time_launches(lambda: dvp.hbm_probe(mode, b["zt"], b["zi"], b["dz"]), 10, 2)
            return median(pl)
        mat = n * v * elem
        t_read, t_fill, t_rows = probe(dvp.PROBE_READ), probe(dvp.PROBE_FILL), probe(dvp.PROBE_ROWS_2R1W)
        t_wide, t_once = probe(dvp.PROBE_FILL_WIDE), probe(dvp.PROBE_READ_ONESHOT)
        read_gbs, fill_gbs, rows_gbs = 2 * mat / t_read / 1e6, mat / t_fill / 1e6, 3 * mat / t_rows / 1e6
        result["stream_ceiling"] = {
            "what": "streaming kernels without arithmetic over this workload's own matrices (dvp_hbm_probe), median of 10 launches",
            "read_two_matrices_gbs": read_gbs, "fill_one_matrix_gbs": fill_gbs, "rows_2_reads_1_write_gbs": rows_gbs,
            # the same bytes in other shapes: a fill from 1024-thread workgroups with two plain stores each (slower), and
            # reads by workgroups that take 16 KB and leave (faster; not a shape a kernel that keeps a row in one CU's
            # registers can have)
            "fill_wide_workgroups_gbs": mat / t_wide / 1e6, "read_oneshot_workgroups_gbs": 2 * mat / t_once / 1e6,
            # a call whose row kernel only reads and whose gradient is written by a write-only kernel: 2 parts read, 1 part filled
            "separate_phases_frac_of_peak": 3.0 / (2.0 / read_gbs + 1.0 / fill_gbs) / HBM_PEAK_GBS,
            # a call whose row kernel writes every gradient row itself (dense rows: no pruning, flat logits)
            "interleaved_rows_frac_of_peak": rows_gbs / HBM_PEAK_GBS}

    print(json.dumps(result))
    if parity_out is not None and not parity_out["ok"]:
        print("bench.py: the timed outputs do NOT match the oracle", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
