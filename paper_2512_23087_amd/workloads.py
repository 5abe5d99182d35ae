"""Seeded synthetic workloads for the DVP row path and the LM-head variant.

These generators stand in for the logits a trainer and a rollout engine would
produce (the paper's Sec. 6 setup needs a 14B policy and a dataset that are not
available).  They hold none of the method's arithmetic: only random draws,
dtype rounding and token sampling from a plain softmax.  Both the GPU tests
and the CPU oracle tests draw their inputs here, so the two sides see the same
stored bit patterns.

Every generator is deterministic for a given (config, device type, shape).
Work is done in row chunks so the largest case (32768 x 151936) needs only a
few GB of temporaries beside its outputs.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

BASE_SEED = 0xD5B0
E4M3_MAX = 448.0


@dataclass
class RowWorkload:
    name: str
    z_train: torch.Tensor            # [N, V] fp32 or bf16
    z_infer: torch.Tensor            # [N, V] same dtype
    ids: torch.Tensor                # [N] int64, sampled tokens
    grad_out: Optional[torch.Tensor]  # [N] fp32 or None (forward-only case)
    rhos: List[float]                # thresholds the case is run at (0 = no pruning)
    forced_rows: Optional[torch.Tensor] = None  # bool [N]: id drawn uniformly, not from the softmax
    meta: dict = field(default_factory=dict)


@dataclass
class LmHeadWorkload:
    name: str
    hidden: torch.Tensor    # [N, d] bf16
    w_train: torch.Tensor   # [V, d] bf16
    w_infer: torch.Tensor   # [V, d] bf16, values representable in fp8-e4m3
    ids: torch.Tensor       # [N] int64
    grad_out: torch.Tensor  # [N] fp32
    rhos: List[float]
    meta: dict = field(default_factory=dict)
    # an 8-bit inference engine for the same model (make_lmhead(f8_engine=True)): activations and head
    # as float8_e4m3fn with per-tensor factors; its logits are scale_infer * hidden8 w8^T
    hidden8: Optional[torch.Tensor] = None
    w8: Optional[torch.Tensor] = None
    scale_infer: float = 1.0


# (N, V, dtype, kind) of the five cases; kind selects the logit recipe below.
ROW_CONFIGS = {
    0: dict(n=64, v=32000, dtype=torch.float32, kind="spikes", infer_sigma=0.02,
            fp8_infer=False, temperature=1.0, backward=False, rhos=[1e-4]),
    1: dict(n=2048, v=32000, dtype=torch.bfloat16, kind="spikes", infer_sigma=0.02,
            fp8_infer=True, temperature=1.0, backward=True, rhos=[1e-4]),
    2: dict(n=8192, v=151936, dtype=torch.bfloat16, kind="student_t", infer_sigma=0.01,
            fp8_infer=False, temperature=1.0, backward=True, forced_every=20,
            rhos=[1e-4, math.exp(-13.0)]),
    3: dict(n=32768, v=151936, dtype=torch.bfloat16, kind="student_t", infer_sigma=0.01,
            fp8_infer=False, temperature=0.7, backward=True, forced_every=20,
            rhos=[1e-2, 1e-4, 1e-6, 0.0]),
}
LMHEAD_CONFIG = dict(n=16384, d=4096, v=151936, w_sigma=0.02, rhos=[1e-4, math.exp(-13.0)])


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def through_e4m3(x: torch.Tensor) -> torch.Tensor:
    """Round fp32 values to the fp8-e4m3 (finite, max 448) grid and return
    them as fp32; saturating, round-to-nearest-even."""
    return x.clamp(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn).to(torch.float32)


def _sample_ids(z_infer_chunk: torch.Tensor, g) -> torch.Tensor:
    """Draw one token per row from the plain softmax of the stored inference
    logits (fp64, inverse CDF)."""
    p = torch.softmax(z_infer_chunk.to(torch.float64), dim=-1)
    cdf = torch.cumsum(p, dim=-1)
    u = torch.rand(p.shape[0], 1, generator=g, device=p.device, dtype=torch.float64)
    idx = (cdf < u * cdf[:, -1:]).sum(dim=-1)
    return idx.clamp_(max=p.shape[1] - 1)


def make_rows(config: int, device="cpu", n: Optional[int] = None, v: Optional[int] = None,
              chunk: int = 512) -> RowWorkload:
    """Build row-path case `config` (0..3).  `n` / `v` override the shape for
    reduced-size parity cases; the recipe stays the same."""
    c = dict(ROW_CONFIGS[config])
    n = c["n"] if n is None else n
    v = c["v"] if v is None else v
    dev = torch.device(device)
    g = _gen(dev, BASE_SEED + config)
    dt = c["dtype"]
    z_train = torch.empty(n, v, dtype=dt, device=dev)
    z_infer = torch.empty(n, v, dtype=dt, device=dev)
    ids = torch.empty(n, dtype=torch.int64, device=dev)
    forced = None
    if c.get("forced_every"):
        forced = (torch.arange(n, device=dev) % c["forced_every"]) == 0

    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        m = r1 - r0
        if c["kind"] == "spikes":
            # N(0, 2^2) base; 5 distinct positions per row overwritten with U[8, 12]
            base = 2.0 * torch.randn(m, v, generator=g, device=dev)
            n_spk = min(5, v)
            keys = torch.rand(m, v, generator=g, device=dev)
            pos = keys.topk(n_spk, dim=-1).indices
            val = 8.0 + 4.0 * torch.rand(m, n_spk, generator=g, device=dev)
            base.scatter_(1, pos, val)
        else:
            # Student-t with 3 degrees of freedom, scale 2, divided by the temperature
            num = torch.randn(m, v, generator=g, device=dev)
            den = torch.zeros(m, v, device=dev)
            for _ in range(3):
                den += torch.randn(m, v, generator=g, device=dev) ** 2
            base = 2.0 * num / torch.sqrt(den / 3.0) / c["temperature"]
            del num, den
        tr = base.to(dt)
        # the inference engine sees the trainer's (stored) logits plus bounded noise
        inf = tr.to(torch.float32) + c["infer_sigma"] * torch.randn(m, v, generator=g, device=dev)
        if c["fp8_infer"]:
            inf = through_e4m3(inf)
        inf = inf.to(dt)
        z_train[r0:r1] = tr
        z_infer[r0:r1] = inf
        ids[r0:r1] = _sample_ids(inf, g)
        del base, tr, inf

    if forced is not None:
        # these rows take a uniformly drawn token instead: with heavy-tailed
        # logits almost every token is far below the row maximum
        uni = torch.randint(0, v, (n,), generator=g, device=dev)
        ids = torch.where(forced, uni, ids)
    grad_out = torch.randn(n, generator=g, device=dev) if c["backward"] else None
    return RowWorkload(name="rows_cfg%d_N%d_V%d_%s" % (config, n, v, str(dt).split(".")[-1]),
                       z_train=z_train, z_infer=z_infer, ids=ids, grad_out=grad_out,
                       rhos=list(c["rhos"]), forced_rows=forced,
                       meta=dict(config=config, n=n, v=v))


def make_lmhead(device="cpu", n: Optional[int] = None, d: Optional[int] = None,
                v: Optional[int] = None, chunk: int = 1024, f8_engine: bool = False,
                hidden_scale: float = 1.0, flat_every: int = 0) -> LmHeadWorkload:
    """Hidden states ~ N(0,1), head weights ~ N(0, 0.02^2), both bf16; the
    inference head is the same matrix rounded through fp8-e4m3.  Tokens are
    sampled from the softmax of the inference logits H W_infer^T.

    hidden_scale: the hidden states are multiplied by it.  At 1 the logits have
    a standard deviation of 0.02 sqrt(d) (1.28 at d = 4096) and nearly every
    token is within log(1e-4) of the row maximum; at 20 they are peaked the way
    a trained model's are, and a row's safe set at rho = 1e-4 is a few tokens.
    flat_every = k > 0: every k-th row keeps the scale 1 (a batch of peaked rows
    with flat, high-entropy ones among them).

    f8_engine: the inference side is instead an 8-bit engine: activations
    e4m3(H / s_h) and head e4m3(W / s_w) with per-tensor factors s = max|.| / 448
    (the usual per-tensor FP8 recipe), logits (s_h s_w) * hidden8 w8^T, and the
    tokens are sampled from those."""
    c = LMHEAD_CONFIG
    n = c["n"] if n is None else n
    d = c["d"] if d is None else d
    v = c["v"] if v is None else v
    dev = torch.device(device)
    g = _gen(dev, BASE_SEED + 4)
    h32 = torch.randn(n, d, generator=g, device=dev)
    row_scale = torch.full((n, 1), float(hidden_scale), device=dev)
    if flat_every > 0:
        row_scale[::flat_every] = 1.0
    hidden = (row_scale * h32).to(torch.bfloat16)
    del h32, row_scale
    w32 = c["w_sigma"] * torch.randn(v, d, generator=g, device=dev)
    w_train = w32.to(torch.bfloat16)
    w_infer = through_e4m3(w_train.to(torch.float32)).to(torch.bfloat16)
    del w32
    ids = torch.empty(n, dtype=torch.int64, device=dev)
    mm_dtype = torch.float32
    hidden8 = w8 = None
    scale_infer = 1.0
    if f8_engine:
        s_h = float(hidden.float().abs().max().item()) / E4M3_MAX
        s_w = float(w_train.float().abs().max().item()) / E4M3_MAX
        hidden8 = (hidden.float() / s_h).clamp(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn)
        w8 = torch.empty(v, d, dtype=torch.float8_e4m3fn, device=dev)
        for r0 in range(0, v, 16384):
            w8[r0:r0 + 16384] = (w_train[r0:r0 + 16384].float() / s_w).clamp(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn)
        scale_infer = float(torch.tensor(s_h * s_w, dtype=torch.float32).item())   # the fp32 value both sides use
        lhs, wi = hidden8, w8.to(mm_dtype)
    else:
        lhs, wi = hidden, w_infer.to(mm_dtype)
    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        logits = scale_infer * (lhs[r0:r1].to(mm_dtype) @ wi.T)
        ids[r0:r1] = _sample_ids(logits, g)
        del logits
    del wi
    grad_out = torch.randn(n, generator=g, device=dev)
    return LmHeadWorkload(name="lmhead_N%d_d%d_V%d" % (n, d, v), hidden=hidden,
                          w_train=w_train, w_infer=w_infer, ids=ids, grad_out=grad_out,
                          rhos=list(c["rhos"]), meta=dict(n=n, d=d, v=v), hidden8=hidden8, w8=w8,
                          scale_infer=scale_infer)
