"""Python face of the fp64 CPU oracle for Dynamic Vocabulary Pruning.

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's CPU-baseline leg; never by the product package.  The arithmetic
lives in ``dvp_oracle.c`` (plain C, double precision); this module compiles it
with gcc, marshals numpy arrays into it and adds the dense LM-head wrapper,
whose only extra steps are three fp64 matrix products.

Parity status: every function here is pinned by tests/test_oracle_pins.py.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "dvp_oracle.c"
_LIB = _HERE / "libdvp_oracle.so"
_lib = None

F32, BF16, F64, F8E4M3 = 0, 1, 2, 3


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
             "-o", str(tmp), str(_SRC), "-lm", "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        alt = os.environ.get("DVP_ORACLE_SRC")   # tests plant mistakes in a copy of the C source,
        if alt:                                  # or build it with other flags (DVP_ORACLE_CFLAGS: sanitizers)
            out = Path(alt).with_suffix(".so")
            extra = os.environ.get("DVP_ORACLE_CFLAGS", "").split()
            subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", *extra,
                                   "-o", str(out), alt, "-lm", "-lpthread"])
            path = out
        else:
            build()
            path = _LIB
        lib = ctypes.CDLL(str(path))
        lib.dvp_oracle_rows.restype = ctypes.c_int
        lib.dvp_oracle_rows.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_float, ctypes.c_double, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        lib.dvp_oracle_rows_finite_mask.restype = ctypes.c_int
        lib.dvp_oracle_rows_finite_mask.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
            ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.dvp_oracle_e4m3_value.restype = ctypes.c_double
        lib.dvp_oracle_e4m3_value.argtypes = [ctypes.c_uint8]
        lib.dvp_oracle_sequences.restype = ctypes.c_int
        lib.dvp_oracle_sequences.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def log_rho_f32(rho: float) -> np.float32:
    """The single fp32 constant log(rho) used by the threshold (App. A,
    protocol item 2).  rho = 0 stands for "no pruning" and maps to -inf."""
    if rho == 0.0:
        return np.float32(-np.inf)
    if not (0.0 < rho <= 1.0):
        raise ValueError("rho must lie in [0, 1]")
    return np.float32(math.log(rho))


def as_oracle_input(z):
    """Accepts a numpy float32/float64/uint16(bf16 bits)/uint8(E4M3 codes) array
    or a CPU torch tensor (float32, float64, bfloat16, float8_e4m3fn); returns
    (array, dtype_code) without changing any stored value."""
    if not isinstance(z, np.ndarray):
        import torch  # plumbing only: reinterpret bf16 / fp8 storage as integers
        t = z.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            z = t.view(torch.int16).numpy().view(np.uint16)
        elif t.dtype == torch.float8_e4m3fn:
            z = t.view(torch.uint8).numpy()
        else:
            z = t.numpy()
    if z.dtype == np.float32:
        code = F32
    elif z.dtype == np.uint16:
        code = BF16
    elif z.dtype == np.float64:
        code = F64
    elif z.dtype == np.uint8:
        code = F8E4M3
    else:
        raise TypeError("unsupported logits dtype %s" % z.dtype)
    if z.ndim != 2:
        raise ValueError("logits must be [N, V]")
    return np.ascontiguousarray(z), code


def e4m3_value(code: int) -> float:
    """Value of one 8-bit E4M3 code (NaN for the two NaN codes)."""
    return float(_load().dvp_oracle_e4m3_value(int(code) & 0xFF))


def rows(z, ids, log_rho, grad_out=None, want_flags=False, want_dz=False,
         band=1e-6, threads=1, want_entropy=False):
    """One side of the DVP forward (and, with want_dz, the gradient of the
    sampled token's constrained log-probability) for every row of z.

    Returns a dict of numpy arrays: row_max, tau, lse_safe, lse_full, logp
    (float64 [N]); safe_count, band_count (int64 [N]); y_in_safe (uint8 [N]);
    optionally safe_flags (uint8 [N, V]), dz (float64 [N, V]) and entropy (float64 [N]: entropy of
    the constrained policy)."""
    z, code = as_oracle_input(z)
    n, v = z.shape
    ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int64))
    if ids.shape != (n,):
        raise ValueError("ids must be [N]")
    g = None
    if grad_out is not None:
        g = np.ascontiguousarray(np.asarray(grad_out, dtype=np.float64))
        if g.shape != (n,):
            raise ValueError("grad_out must be [N]")
    out = {
        "row_max": np.empty(n, np.float64), "tau": np.empty(n, np.float64),
        "lse_safe": np.empty(n, np.float64), "lse_full": np.empty(n, np.float64),
        "logp": np.empty(n, np.float64),
        "safe_count": np.empty(n, np.int64), "band_count": np.empty(n, np.int64),
        "y_in_safe": np.empty(n, np.uint8),
    }
    flags = np.empty((n, v), np.uint8) if want_flags else None
    dz = np.empty((n, v), np.float64) if want_dz else None
    ent = np.empty(n, np.float64) if want_entropy else None

    def p(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().dvp_oracle_rows(
        p(z), code, n, v, v, p(ids), ctypes.c_float(float(log_rho)), float(band), p(g),
        p(out["row_max"]), p(out["tau"]), p(out["lse_safe"]), p(out["lse_full"]),
        p(out["logp"]), p(out["safe_count"]), p(out["band_count"]), p(out["y_in_safe"]),
        p(flags), p(dz), int(threads), p(ent))
    if rc != 0:
        raise RuntimeError("dvp_oracle_rows failed with code %d" % rc)
    if want_flags:
        out["safe_flags"] = flags
    if want_dz:
        out["dz"] = dz
    if want_entropy:
        out["entropy"] = ent
    return out


def rows_finite_mask(z, ids, log_rho, mask_value=-50.0, grad_out=None, want_flags=False, want_dz=False):
    """The finite-mask variant (Sec. 5.5 "Logit Masking Strategy", App. A item 3): pruned logits
    become `mask_value`, the threshold is evaluated in the logits' storage arithmetic, and log-softmax
    runs over the whole masked row.  `log_rho` is the double log(rho).  Returns row_max, tau, lse, logp
    (float64 [N]), safe_count (int64 [N]), y_in_safe (uint8 [N]), optionally safe_flags and dz."""
    z, code = as_oracle_input(z)
    if code == F8E4M3:
        raise TypeError("8-bit logits are an inference-side format of the exact path only")
    n, v = z.shape
    ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int64))
    g = None if grad_out is None else np.ascontiguousarray(np.asarray(grad_out, dtype=np.float64))
    out = {"row_max": np.empty(n, np.float64), "tau": np.empty(n, np.float64), "lse": np.empty(n, np.float64),
           "logp": np.empty(n, np.float64), "safe_count": np.empty(n, np.int64), "y_in_safe": np.empty(n, np.uint8)}
    flags = np.empty((n, v), np.uint8) if want_flags else None
    dz = np.empty((n, v), np.float64) if want_dz else None

    def p(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().dvp_oracle_rows_finite_mask(p(z), code, n, v, v, p(ids), float(log_rho), float(mask_value), p(g),
                                             p(out["row_max"]), p(out["tau"]), p(out["lse"]), p(out["logp"]),
                                             p(out["safe_count"]), p(out["y_in_safe"]), p(flags), p(dz))
    if rc != 0:
        raise RuntimeError("dvp_oracle_rows_finite_mask failed with code %d" % rc)
    if want_flags:
        out["safe_flags"] = flags
    if want_dz:
        out["dz"] = dz
    return out


def _widen(a):
    """Exact widening of a stored matrix (numpy f32/f64/bf16-bits or torch)."""
    a, code = as_oracle_input(a)
    if code == BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if code == F8E4M3:
        table = np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)
        return table[a]
    return a.astype(np.float64)


def lmhead(hidden, w, ids, log_rho, grad_out=None, want_flags=False, band=1e-6, threads=1, scale=1.0):
    """Dense LM-head variant: logits z = scale * H W^T formed in fp64 from the
    stored hidden states H [N, d] and head weights W [V, d] (bf16, fp32 or, for
    an 8-bit inference engine as in Sec. 4.2, E4M3 codes with `scale` the
    product of its two dequantisation factors), then ``rows`` on them; with
    grad_out also dH = dz W and dW = dz^T H (chain rule through the linear map;
    scale must be 1 there).  Returns the ``rows`` dict plus 'z', and
    'd_hidden', 'd_w' when grad_out is given."""
    h64 = _widen(hidden)
    w64 = _widen(w)
    if grad_out is not None and scale != 1.0:
        raise ValueError("the gradient is defined for the training side only (scale = 1)")
    z = float(scale) * (h64 @ w64.T)
    out = rows(z, ids, log_rho, grad_out=grad_out, want_flags=want_flags,
               want_dz=grad_out is not None, band=band, threads=threads)
    out["z"] = z
    if grad_out is not None:
        out["d_hidden"] = out["dz"] @ w64
        out["d_w"] = out["dz"].T @ h64
    return out


def log_threshold_f32(threshold: float) -> np.float32:
    """The single fp32 constant log(threshold) the token veto compares with
    (App. A, protocol item 5; threshold 1e-4 in the paper)."""
    if not (threshold > 0.0):
        raise ValueError("threshold must be positive")
    return np.float32(math.log(threshold))


def sequences(logp_train, logp_infer, offsets, log_threshold):
    """Sequence-level importance weights and token veto (Thm. 4.1; App. A
    protocol items 4 and 5) from the two sides' fp32 constrained log-probs.
    offsets: int64 [n_seq + 1]; sequence s owns tokens offsets[s] .. offsets[s+1]-1.
    Returns weight (float64 [N], NaN where no sequence owns the token),
    seq_log_ratio, seq_min_weight (float64 [n_seq]), seq_veto (uint8 [n_seq])."""
    lt = np.ascontiguousarray(np.asarray(logp_train, dtype=np.float32))
    li = np.ascontiguousarray(np.asarray(logp_infer, dtype=np.float32))
    off = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
    n, n_seq = lt.shape[0], off.shape[0] - 1
    if li.shape != (n,) or n_seq < 0:
        raise ValueError("shape mismatch")
    out = {"weight": np.full(n, np.nan, np.float64), "seq_log_ratio": np.empty(n_seq, np.float64),
           "seq_min_weight": np.empty(n_seq, np.float64), "seq_veto": np.empty(n_seq, np.uint8)}

    def p(a):
        return a.ctypes.data_as(ctypes.c_void_p)

    rc = _load().dvp_oracle_sequences(n, n_seq, p(lt), p(li), p(off), ctypes.c_float(float(log_threshold)),
                                      p(out["weight"]), p(out["seq_log_ratio"]), p(out["seq_min_weight"]),
                                      p(out["seq_veto"]))
    if rc != 0:
        raise RuntimeError("dvp_oracle_sequences failed with code %d" % rc)
    return out
