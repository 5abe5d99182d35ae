"""Thin ctypes binding over the C-ABI library `libdvp_hip.so`.

Argument marshalling only: tensors supply device memory and the current
stream, every step of the computation runs in the HIP kernels.  There is no
CPU or PyTorch fallback: a missing or unloadable library raises ImportError
at first use, and calls on non-GPU tensors raise.
"""
from __future__ import annotations

import ctypes
import math
from pathlib import Path
from typing import Optional

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libdvp_hip.so"

DVP_F32, DVP_BF16, DVP_F8E4M3 = 0, 1, 2
ROW_Y_IN_TRAIN_SAFE, ROW_Y_IN_INFER_SAFE, ROW_ID_OUT_OF_RANGE, ROW_GRAD_OVERFLOW, ROW_SHORT_SAFE_SET = 1, 2, 4, 8, 16
SHORT_SAFE_SET_MAX = 64

EXPORTS = ("dvp_forward", "dvp_backward", "dvp_forward_backward", "dvp_fused_lmhead",
           "dvp_fused_lmhead_workspace_bytes", "dvp_log_rho", "dvp_status_string", "dvp_row_path",
           "dvp_sequence_weights", "dvp_log_threshold", "dvp_forward_backward_sparse",
           "dvp_fused_lmhead_f8infer", "dvp_lists_to_dense", "dvp_fused_lmhead_saved_bytes",
           "dvp_fused_lmhead_forward", "dvp_fused_lmhead_backward", "dvp_fused_lmhead_lists",
           "dvp_fused_lmhead_lists_workspace_bytes", "dvp_fused_lmhead_lists_second_pass_rows",
           "dvp_fused_lmhead_lists_f8infer", "dvp_fused_lmhead_rows", "dvp_fused_lmhead_rows_workspace_bytes",
           "dvp_prepare", "dvp_fused_lmhead_forward_noalloc", "dvp_hbm_probe",
           "dvp_fused_lmhead_select_rows", "dvp_fused_lmhead_rows_counted", "dvp_set_split_min_bytes")


class DvpParams(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("vocab", ctypes.c_int64),
                ("ld_train", ctypes.c_int64), ("ld_infer", ctypes.c_int64),
                ("ld_grad", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("log_rho", ctypes.c_float), ("dtype_infer", ctypes.c_int32),
                ("mode", ctypes.c_int32), ("mask_value", ctypes.c_float)]


class DvpSideOut(ctypes.Structure):
    _fields_ = [("logp", ctypes.c_void_p), ("row_max", ctypes.c_void_p),
                ("lse_safe", ctypes.c_void_p), ("lse_full", ctypes.c_void_p),
                ("safe_count", ctypes.c_void_p), ("safe_bits", ctypes.c_void_p),
                ("entropy", ctypes.c_void_p)]


class DvpLmHeadParams(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("hidden", ctypes.c_int64), ("vocab", ctypes.c_int64),
                ("ld_hidden", ctypes.c_int64), ("ld_w", ctypes.c_int64),
                ("log_rho", ctypes.c_float)]


class DvpLmHeadF8Side(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_void_p), ("w", ctypes.c_void_p), ("ld_hidden", ctypes.c_int64),
                ("ld_w", ctypes.c_int64), ("scale", ctypes.c_float)]


class DvpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib():
    """Load the shared library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError("%s not found: run `python -m paper_2512_23087_amd.build` "
                              "(there is no fallback path)" % LIB_PATH)
        L = ctypes.CDLL(str(LIB_PATH))
        vp, i64p = ctypes.c_void_p, ctypes.c_void_p
        pp, sp = ctypes.POINTER(DvpParams), ctypes.POINTER(DvpSideOut)
        L.dvp_forward.restype = ctypes.c_int
        L.dvp_forward.argtypes = [pp, vp, vp, i64p, sp, sp, vp, vp]
        L.dvp_backward.restype = ctypes.c_int
        L.dvp_backward.argtypes = [pp, vp, i64p, vp, vp, vp, vp, vp, vp]
        L.dvp_forward_backward.restype = ctypes.c_int
        L.dvp_forward_backward.argtypes = [pp, vp, vp, i64p, vp, sp, sp, vp, vp, vp]
        lp = ctypes.POINTER(DvpLmHeadParams)
        L.dvp_fused_lmhead_workspace_bytes.restype = ctypes.c_size_t
        L.dvp_fused_lmhead_workspace_bytes.argtypes = [lp]
        L.dvp_fused_lmhead.restype = ctypes.c_int
        L.dvp_fused_lmhead.argtypes = [lp, vp, vp, vp, i64p, vp, sp, sp, vp, vp, vp, vp,
                                       ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_f8infer.restype = ctypes.c_int
        L.dvp_fused_lmhead_f8infer.argtypes = [lp, vp, vp, ctypes.POINTER(DvpLmHeadF8Side), i64p, vp, sp, sp, vp, vp,
                                               vp, vp, ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_saved_bytes.restype = ctypes.c_size_t
        L.dvp_fused_lmhead_saved_bytes.argtypes = [lp]
        L.dvp_fused_lmhead_forward.restype = ctypes.c_int
        L.dvp_fused_lmhead_forward.argtypes = [lp, vp, vp, vp, ctypes.POINTER(DvpLmHeadF8Side), i64p, sp, sp, vp, vp,
                                               ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_backward.restype = ctypes.c_int
        L.dvp_fused_lmhead_backward.argtypes = [lp, vp, vp, i64p, vp, vp, ctypes.c_size_t, vp, vp, vp,
                                                ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_lists_workspace_bytes.restype = ctypes.c_size_t
        L.dvp_fused_lmhead_lists_workspace_bytes.argtypes = [lp, ctypes.c_int32]
        L.dvp_fused_lmhead_lists_second_pass_rows.restype = ctypes.c_size_t
        L.dvp_fused_lmhead_lists_second_pass_rows.argtypes = [lp, ctypes.c_int32]
        L.dvp_fused_lmhead_lists.restype = ctypes.c_int
        L.dvp_fused_lmhead_lists.argtypes = [lp, vp, vp, vp, i64p, vp, sp, sp, vp, vp, vp, ctypes.c_int32, vp, vp, vp,
                                             ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_lists_f8infer.restype = ctypes.c_int
        L.dvp_fused_lmhead_lists_f8infer.argtypes = [lp, vp, vp, ctypes.POINTER(DvpLmHeadF8Side), i64p, vp, sp, sp, vp, vp, vp,
                                                     ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_rows_workspace_bytes.restype = ctypes.c_size_t
        L.dvp_fused_lmhead_rows_workspace_bytes.argtypes = [lp, ctypes.c_int64]
        L.dvp_fused_lmhead_rows.restype = ctypes.c_int
        L.dvp_fused_lmhead_rows.argtypes = [lp, vp, vp, i64p, vp, vp, ctypes.c_int64, vp, vp, vp, ctypes.c_size_t, vp]
        L.dvp_fused_lmhead_select_rows.restype = ctypes.c_int
        L.dvp_fused_lmhead_select_rows.argtypes = [ctypes.c_int64, vp, ctypes.c_uint32, vp, ctypes.c_int64, vp, vp, vp]
        L.dvp_fused_lmhead_rows_counted.restype = ctypes.c_int
        L.dvp_fused_lmhead_rows_counted.argtypes = [lp, vp, vp, i64p, vp, vp, vp, ctypes.c_int64, vp, vp, vp, ctypes.c_size_t, vp]
        L.dvp_log_rho.restype = ctypes.c_float
        L.dvp_log_rho.argtypes = [ctypes.c_double]
        L.dvp_status_string.restype = ctypes.c_char_p
        L.dvp_status_string.argtypes = [ctypes.c_int]
        L.dvp_row_path.restype = ctypes.c_int
        L.dvp_row_path.argtypes = [pp, ctypes.c_int]
        L.dvp_forward_backward_sparse.restype = ctypes.c_int
        L.dvp_forward_backward_sparse.argtypes = [pp, vp, vp, i64p, vp, sp, sp, vp, vp, vp, ctypes.c_int32, vp]
        L.dvp_lists_to_dense.restype = ctypes.c_int
        L.dvp_lists_to_dense.argtypes = [pp, vp, vp, ctypes.c_int32, vp, vp, vp, i64p, vp, vp, vp, vp]
        L.dvp_sequence_weights.restype = ctypes.c_int
        L.dvp_sequence_weights.argtypes = [ctypes.c_int64, ctypes.c_int64, vp, vp, i64p, ctypes.c_float,
                                           vp, vp, vp, vp, vp]
        L.dvp_log_threshold.restype = ctypes.c_float
        L.dvp_log_threshold.argtypes = [ctypes.c_double]
        L.dvp_prepare.restype = ctypes.c_int
        L.dvp_prepare.argtypes = []
        L.dvp_set_split_min_bytes.restype = ctypes.c_int64
        L.dvp_set_split_min_bytes.argtypes = [ctypes.c_int64]
        L.dvp_hbm_probe.restype = ctypes.c_int
        L.dvp_hbm_probe.argtypes = [ctypes.c_int, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, vp]
        L.dvp_fused_lmhead_forward_noalloc.restype = ctypes.c_int
        L.dvp_fused_lmhead_forward_noalloc.argtypes = [lp, vp, vp, vp, i64p, sp, sp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().dvp_status_string(int(status)).decode()


SPLIT_MIN_BYTES_DEFAULT = 512 << 20


def set_split_min_bytes(nbytes: int) -> int:
    """Gradient size from which dvp_forward_backward writes the gradient in two steps; returns the
    previous value (a negative argument only reads it).  See dvp_set_split_min_bytes in dvp.h."""
    return int(lib().dvp_set_split_min_bytes(int(nbytes)))


def prepare() -> None:
    """One-time set-up of every kernel build on the current device (see dvp_prepare in dvp.h)."""
    st = lib().dvp_prepare()
    if st != 0:
        raise DvpError(st, "dvp_prepare")


PROBE_READ, PROBE_FILL, PROBE_ROWS_2R1W, PROBE_FILL_WIDE, PROBE_READ_ONESHOT = 0, 1, 2, 3, 4


def hbm_probe(mode: int, a, b, c, *, stream=None) -> None:
    """A streaming kernel without arithmetic over [N, row] matrices (see dvp_hbm_probe in dvp.h)."""
    ref = c if mode in (PROBE_FILL, PROBE_FILL_WIDE) else a
    st = lib().dvp_hbm_probe(int(mode), _ptr(a), _ptr(b), _ptr(c), ref.shape[0], ref.stride(0) * ref.element_size(),
                             _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_hbm_probe")


def log_rho(rho: float) -> float:
    """(float)log(rho) as the library computes it; rho = 0 -> -inf (no pruning)."""
    return float(lib().dvp_log_rho(float(rho)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DVP_F32
    if t.dtype == torch.bfloat16:
        return DVP_BF16
    raise TypeError("logits must be float32 or bfloat16, got %s" % t.dtype)


def _infer_dtype_code(z_train: torch.Tensor, z_infer: Optional[torch.Tensor]) -> int:
    """Inference logits share the training logits' dtype or are 8-bit E4M3 (torch.float8_e4m3fn)."""
    if z_infer is None or z_infer.dtype == z_train.dtype:
        return _dtype_code(z_train)
    if z_infer.dtype == torch.float8_e4m3fn:
        return DVP_F8E4M3
    raise ValueError("z_infer must have z_train's dtype or be float8_e4m3fn, got %s" % z_infer.dtype)


def _check_pair(z_train, z_infer):
    _check_rows(z_train, "z_train")
    if z_infer is not None:
        _check_rows(z_infer, "z_infer")
        if z_infer.shape != z_train.shape:
            raise ValueError("z_infer must match z_train in shape")
        _infer_dtype_code(z_train, z_infer)


def _check_rows(z: torch.Tensor, name: str):
    if not z.is_cuda:
        raise ValueError("%s must live in GPU memory (no CPU path exists)" % name)
    if z.dim() != 2 or z.stride(1) != 1:
        raise ValueError("%s must be [N, V] with unit stride along V" % name)


class SideOutputs:
    """Device buffers for one side's per-row outputs."""

    def __init__(self, n, vocab, device, lse_full=False, safe_bits=False, entropy=False):
        self.logp = torch.empty(n, dtype=torch.float32, device=device)
        self.row_max = torch.empty(n, dtype=torch.float32, device=device)
        self.lse_safe = torch.empty(n, dtype=torch.float32, device=device)
        self.lse_full = torch.empty(n, dtype=torch.float32, device=device) if lse_full else None
        self.safe_count = torch.empty(n, dtype=torch.int32, device=device)
        self.safe_bits = (torch.empty(n, (vocab + 31) // 32, dtype=torch.int32, device=device)
                          if safe_bits else None)
        self.entropy = torch.empty(n, dtype=torch.float32, device=device) if entropy else None

    def struct(self) -> DvpSideOut:
        return DvpSideOut(*(None if t is None else t.data_ptr() for t in
                            (self.logp, self.row_max, self.lse_safe, self.lse_full,
                             self.safe_count, self.safe_bits, self.entropy)))

    def flags_matrix(self, vocab) -> torch.Tensor:
        """Expand safe_bits to a uint8 [N, V] matrix (test helper; torch ops)."""
        words = self.safe_bits.to(torch.int64) & 0xFFFFFFFF
        shifts = torch.arange(32, device=words.device, dtype=torch.int64)
        bits = ((words.unsqueeze(-1) >> shifts) & 1).to(torch.uint8)
        return bits.reshape(words.shape[0], -1)[:, :vocab]


class RowResult:
    def __init__(self, train: SideOutputs, infer: Optional[SideOutputs], row_flags, dz):
        self.train, self.infer, self.row_flags, self.dz = train, infer, row_flags, dz


DVP_MODE_EXACT, DVP_MODE_FINITE_MASK = 0, 1


def _params(z_train, z_infer, dz, log_rho_value, mask_value=None) -> DvpParams:
    """mask_value not None selects the finite-mask variant (pruned logits count as that constant)."""
    return DvpParams(z_train.shape[0], z_train.shape[1], z_train.stride(0),
                     z_infer.stride(0) if z_infer is not None else 0,
                     dz.stride(0) if dz is not None else 0,
                     _dtype_code(z_train), float(log_rho_value), _infer_dtype_code(z_train, z_infer),
                     DVP_MODE_EXACT if mask_value is None else DVP_MODE_FINITE_MASK,
                     0.0 if mask_value is None else float(mask_value))


def dvp_forward(z_train, z_infer, ids, log_rho_value, *, lse_full=False, safe_bits=False, entropy=False,
                out_train: Optional[SideOutputs] = None, out_infer: Optional[SideOutputs] = None,
                row_flags: Optional[torch.Tensor] = None, stream=None, mask_value=None) -> RowResult:
    _check_pair(z_train, z_infer)
    n, v = z_train.shape
    dev = z_train.device
    out_train = out_train or SideOutputs(n, v, dev, lse_full, safe_bits, entropy)
    if z_infer is not None:
        out_infer = out_infer or SideOutputs(n, v, dev, lse_full, safe_bits, entropy)
    if row_flags is None:
        row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    p = _params(z_train, z_infer, None, log_rho_value, mask_value)
    st = lib().dvp_forward(ctypes.byref(p), _ptr(z_train), _ptr(z_infer), _ptr(ids),
                           ctypes.byref(out_train.struct()),
                           ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                           _ptr(row_flags), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_forward")
    return RowResult(out_train, out_infer, row_flags, None)


def dvp_backward(z_train, ids, grad_out, row_max_train, lse_safe_train, row_flags, log_rho_value,
                 *, dz: Optional[torch.Tensor] = None, stream=None, mask_value=None) -> torch.Tensor:
    _check_rows(z_train, "z_train")
    if dz is None:
        dz = torch.empty_like(z_train)
    p = _params(z_train, None, dz, log_rho_value, mask_value)
    st = lib().dvp_backward(ctypes.byref(p), _ptr(z_train), _ptr(ids), _ptr(grad_out),
                            _ptr(row_max_train), _ptr(lse_safe_train), _ptr(row_flags), _ptr(dz),
                            _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_backward")
    return dz


def dvp_forward_backward(z_train, z_infer, ids, grad_out, log_rho_value, *, lse_full=False,
                         safe_bits=False, entropy=False, out_train: Optional[SideOutputs] = None,
                         out_infer: Optional[SideOutputs] = None,
                         row_flags: Optional[torch.Tensor] = None,
                         dz: Optional[torch.Tensor] = None, stream=None, mask_value=None) -> RowResult:
    _check_pair(z_train, z_infer)
    n, v = z_train.shape
    dev = z_train.device
    out_train = out_train or SideOutputs(n, v, dev, lse_full, safe_bits, entropy)
    if z_infer is not None:
        out_infer = out_infer or SideOutputs(n, v, dev, lse_full, safe_bits, entropy)
    if row_flags is None:
        row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    if dz is None:
        dz = torch.empty_like(z_train)
    p = _params(z_train, z_infer, dz, log_rho_value, mask_value)
    st = lib().dvp_forward_backward(ctypes.byref(p), _ptr(z_train), _ptr(z_infer), _ptr(ids),
                                    _ptr(grad_out), ctypes.byref(out_train.struct()),
                                    ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                    _ptr(row_flags), _ptr(dz), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_forward_backward")
    return RowResult(out_train, out_infer, row_flags, dz)


class SparseResult:
    def __init__(self, train, infer, row_flags, entries, grad_len):
        self.train, self.infer, self.row_flags = train, infer, row_flags
        self.entries, self.grad_len = entries, grad_len      # entries: int32 [N, cap, 2] = (index, fp32 bits)

    def row(self, i):
        """(indices int64, values float32) of row i, sorted by index (host-side test helper)."""
        n = int(self.grad_len[i].item())
        if int(self.row_flags[i].item()) & ROW_GRAD_OVERFLOW:
            return None
        e = self.entries[i, :n].cpu()
        idx = e[:, 0].to(torch.int64) & 0xFFFFFFFF
        val = e[:, 1].contiguous().view(torch.float32)
        order = torch.argsort(idx)
        return idx[order], val[order]


def dvp_forward_backward_sparse(z_train, z_infer, ids, grad_out, log_rho_value, list_cap, *,
                                out_train: Optional[SideOutputs] = None,
                                out_infer: Optional[SideOutputs] = None, row_flags=None, entries=None,
                                grad_len=None, stream=None) -> SparseResult:
    _check_pair(z_train, z_infer)
    n, v = z_train.shape
    dev = z_train.device
    out_train = out_train or SideOutputs(n, v, dev)
    if z_infer is not None:
        out_infer = out_infer or SideOutputs(n, v, dev)
    if row_flags is None:
        row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    if entries is None:
        entries = torch.empty(n, list_cap, 2, dtype=torch.int32, device=dev)
    if grad_len is None:
        grad_len = torch.empty(n, dtype=torch.int32, device=dev)
    p = _params(z_train, z_infer, None, log_rho_value)
    st = lib().dvp_forward_backward_sparse(ctypes.byref(p), _ptr(z_train), _ptr(z_infer), _ptr(ids),
                                           _ptr(grad_out), ctypes.byref(out_train.struct()),
                                           ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                           _ptr(row_flags), _ptr(entries), _ptr(grad_len), int(list_cap),
                                           _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_forward_backward_sparse")
    return SparseResult(out_train, out_infer, row_flags, entries, grad_len)


def dvp_lists_to_dense(sparse: SparseResult, vocab, dtype, grad_out=None, log_rho_value=-1.0, *, z_train=None,
                       ids=None, dz: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Dense [N, vocab] gradient of `dtype` from the lists of dvp_forward_backward_sparse, scaled row by
    row with grad_out.  With z_train (and ids) the rows whose list overflowed are computed from the logits."""
    n, cap = sparse.entries.shape[0], sparse.entries.shape[1]
    dev = sparse.entries.device
    if dz is None:
        dz = torch.empty(n, vocab, dtype=dtype, device=dev)
    code = DVP_F32 if dz.dtype == torch.float32 else DVP_BF16
    if dz.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("dz must be float32 or bfloat16")
    p = DvpParams(n, vocab, z_train.stride(0) if z_train is not None else vocab, 0, dz.stride(0), code,
                  float(log_rho_value), code, DVP_MODE_EXACT, 0.0)
    st = lib().dvp_lists_to_dense(ctypes.byref(p), _ptr(sparse.entries), _ptr(sparse.grad_len), int(cap),
                                  _ptr(sparse.row_flags), _ptr(grad_out), _ptr(z_train), _ptr(ids),
                                  _ptr(sparse.train.row_max) if z_train is not None else None,
                                  _ptr(sparse.train.lse_safe) if z_train is not None else None, _ptr(dz),
                                  _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_lists_to_dense")
    return dz


class LmHeadResult:
    def __init__(self, train, infer, row_flags, d_hidden, d_w):
        self.train, self.infer, self.row_flags = train, infer, row_flags
        self.d_hidden, self.d_w = d_hidden, d_w


def lmhead_workspace_bytes(n, d, v, ld_hidden=None, ld_w=None) -> int:
    p = DvpLmHeadParams(n, d, v, ld_hidden or d, ld_w or d, -1.0)
    return int(lib().dvp_fused_lmhead_workspace_bytes(ctypes.byref(p)))


def dvp_fused_lmhead(hidden, w_train, w_infer, ids, grad_out, log_rho_value, *, lse_full=False, safe_bits=False,
                     workspace: Optional[torch.Tensor] = None, d_hidden=None, d_w=None,
                     stream=None, infer_f8=None) -> LmHeadResult:
    """infer_f8 = (hidden8, w8, scale): the inference side is an 8-bit engine with float8_e4m3fn
    activations [N, d] and head [V, d], logits scale * hidden8 w8^T (then w_infer must be None)."""
    for name, t in (("hidden", hidden), ("w_train", w_train)):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("%s must be a bf16 [rows, d] GPU tensor with unit inner stride" % name)
    if infer_f8 is not None:
        if w_infer is not None:
            raise ValueError("give either w_infer or infer_f8")
        for name, t in (("infer_f8 hidden", infer_f8[0]), ("infer_f8 w", infer_f8[1])):
            if not t.is_cuda or t.dtype != torch.float8_e4m3fn or t.dim() != 2 or t.stride(1) != 1:
                raise ValueError("%s must be a float8_e4m3fn [rows, d] GPU tensor with unit inner stride" % name)
    n, d = hidden.shape
    v = w_train.shape[0]
    dev = hidden.device
    p = DvpLmHeadParams(n, d, v, hidden.stride(0), w_train.stride(0), float(log_rho_value))
    need = int(lib().dvp_fused_lmhead_workspace_bytes(ctypes.byref(p)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    out_train = SideOutputs(n, v, dev, lse_full, safe_bits)
    out_infer = SideOutputs(n, v, dev, lse_full, safe_bits) if (w_infer is not None or infer_f8 is not None) else None
    row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    if grad_out is not None:
        if d_hidden is None:
            d_hidden = torch.empty(n, hidden.stride(0), dtype=torch.float32, device=dev)[:, :d]
        if d_w is None:
            d_w = torch.empty(v, w_train.stride(0), dtype=torch.float32, device=dev)[:, :d]
    if infer_f8 is not None:
        h8, w8, scale = infer_f8
        side = DvpLmHeadF8Side(h8.data_ptr(), w8.data_ptr(), h8.stride(0), w8.stride(0), float(scale))
        st = lib().dvp_fused_lmhead_f8infer(ctypes.byref(p), _ptr(hidden), _ptr(w_train), ctypes.byref(side),
                                            _ptr(ids), _ptr(grad_out), ctypes.byref(out_train.struct()),
                                            ctypes.byref(out_infer.struct()), _ptr(row_flags), _ptr(d_hidden),
                                            _ptr(d_w), _ptr(workspace), workspace.numel(), _stream(stream))
        if st != 0:
            raise DvpError(st, "dvp_fused_lmhead_f8infer")
        return LmHeadResult(out_train, out_infer, row_flags, d_hidden, d_w)
    st = lib().dvp_fused_lmhead(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(w_infer),
                                _ptr(ids), _ptr(grad_out), ctypes.byref(out_train.struct()),
                                ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                _ptr(row_flags), _ptr(d_hidden), _ptr(d_w), _ptr(workspace),
                                workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead")
    return LmHeadResult(out_train, out_infer, row_flags, d_hidden, d_w)


NOALLOC_SCRATCH_BYTES = 64 << 20


def dvp_fused_lmhead_forward_noalloc(hidden, w_train, w_infer, ids, log_rho_value, out_train: SideOutputs,
                                     out_infer: Optional[SideOutputs], row_flags, *, stream=None) -> LmHeadResult:
    """Forward of both sides with the library's own scratch buffer instead of a workspace; every output
    buffer comes from the caller, so nothing is allocated here either."""
    p = DvpLmHeadParams(hidden.shape[0], hidden.shape[1], w_train.shape[0], hidden.stride(0), w_train.stride(0),
                        float(log_rho_value))
    st = lib().dvp_fused_lmhead_forward_noalloc(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(w_infer), _ptr(ids),
                                                ctypes.byref(out_train.struct()),
                                                ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                                _ptr(row_flags), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_forward_noalloc")
    return LmHeadResult(out_train, out_infer, row_flags, None, None)


class LmHeadListsResult(LmHeadResult):
    def __init__(self, train, infer, row_flags, d_hidden, d_w, entries, grad_len):
        super().__init__(train, infer, row_flags, d_hidden, d_w)
        self.entries, self.grad_len = entries, grad_len      # entries: int32 [N, cap, 2] = (token, fp32 bits)

    row = SparseResult.row


def dvp_fused_lmhead_lists(hidden, w_train, w_infer, ids, grad_out, log_rho_value, list_cap, *, lse_full=False,
                           workspace: Optional[torch.Tensor] = None, d_hidden=None, d_w=None, entries=None,
                           grad_len=None, stream=None, infer_f8=None) -> LmHeadListsResult:
    """LM-head variant with the gradient kept as per-row lists (short safe sets).  grad_out None: the
    forward of both sides only."""
    for name, t in (("hidden", hidden), ("w_train", w_train)):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("%s must be a bf16 [rows, d] GPU tensor with unit inner stride" % name)
    n, d = hidden.shape
    v = w_train.shape[0]
    dev = hidden.device
    p = DvpLmHeadParams(n, d, v, hidden.stride(0), w_train.stride(0), float(log_rho_value))
    need = int(lib().dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(p), int(list_cap)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    out_train = SideOutputs(n, v, dev, lse_full, False)
    if infer_f8 is not None and w_infer is not None:
        raise ValueError("give either w_infer or infer_f8")
    out_infer = SideOutputs(n, v, dev, lse_full, False) if (w_infer is not None or infer_f8 is not None) else None
    row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    if grad_out is not None:
        if d_hidden is None:
            d_hidden = torch.empty(n, hidden.stride(0), dtype=torch.float32, device=dev)[:, :d]
        if d_w is None:
            d_w = torch.empty(v, w_train.stride(0), dtype=torch.float32, device=dev)[:, :d]
        if entries is None:
            entries = torch.empty(n, max(int(list_cap), 1), 2, dtype=torch.int32, device=dev)
        if grad_len is None:
            grad_len = torch.empty(n, dtype=torch.int32, device=dev)
    if infer_f8 is not None:
        h8, w8, scale = infer_f8
        for name, t in (("infer_f8 hidden", h8), ("infer_f8 w", w8)):
            if not t.is_cuda or t.dtype != torch.float8_e4m3fn or t.dim() != 2 or t.stride(1) != 1:
                raise ValueError("%s must be a float8_e4m3fn [rows, d] GPU tensor with unit inner stride" % name)
        side = DvpLmHeadF8Side(h8.data_ptr(), w8.data_ptr(), h8.stride(0), w8.stride(0), float(scale))
        st = lib().dvp_fused_lmhead_lists_f8infer(ctypes.byref(p), _ptr(hidden), _ptr(w_train), ctypes.byref(side),
                                                  _ptr(ids), _ptr(grad_out), ctypes.byref(out_train.struct()),
                                                  ctypes.byref(out_infer.struct()), _ptr(row_flags), _ptr(entries),
                                                  _ptr(grad_len), int(list_cap), _ptr(d_hidden), _ptr(d_w),
                                                  _ptr(workspace), workspace.numel(), _stream(stream))
    else:
        st = lib().dvp_fused_lmhead_lists(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(w_infer), _ptr(ids),
                                          _ptr(grad_out), ctypes.byref(out_train.struct()),
                                          ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                          _ptr(row_flags), _ptr(entries), _ptr(grad_len), int(list_cap),
                                          _ptr(d_hidden), _ptr(d_w), _ptr(workspace), workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_lists")
    res = LmHeadListsResult(out_train, out_infer, row_flags, d_hidden, d_w, entries, grad_len)
    off = int(lib().dvp_fused_lmhead_lists_second_pass_rows(ctypes.byref(p), int(list_cap)))
    res.second_pass = workspace[off:off + 8].view(torch.int32)      # device int32 [2]: rows of each side that needed a second pass
    return res


def dvp_fused_lmhead_rows(hidden, w_train, ids, grad_out, log_rho_value, rows, d_hidden, d_w, *,
                          workspace: Optional[torch.Tensor] = None, stream=None):
    """Dense gradient of the token rows listed in `rows` (int32, device): d_hidden[rows] overwritten, d_w += ."""
    n, d = hidden.shape
    v = w_train.shape[0]
    if rows.dtype != torch.int32 or not rows.is_cuda or rows.dim() != 1:
        raise ValueError("rows must be a 1-D int32 GPU tensor")
    p = DvpLmHeadParams(n, d, v, hidden.stride(0), w_train.stride(0), float(log_rho_value))
    n_sub = rows.numel()
    if workspace is None:
        need = int(lib().dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(p), n_sub))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=hidden.device)
    st = lib().dvp_fused_lmhead_rows(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(ids), _ptr(grad_out), _ptr(rows),
                                     n_sub, _ptr(d_hidden), _ptr(d_w), _ptr(workspace), workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_rows")


def dvp_fused_lmhead_select_rows(row_flags, mask, rows, n_sub, *, n_flagged=None, stream=None):
    """rows (int32 [max_rows], device) <- the rows whose flags meet `mask`, ascending, padded with -1;
    n_sub (int32 [1], device) <- how many of them are in rows; n_flagged (optional) <- how many there are."""
    st = lib().dvp_fused_lmhead_select_rows(row_flags.numel(), _ptr(row_flags), int(mask), _ptr(rows), rows.numel(),
                                            _ptr(n_sub), _ptr(n_flagged), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_select_rows")


def dvp_fused_lmhead_rows_counted(hidden, w_train, ids, grad_out, log_rho_value, rows, n_sub, d_hidden, d_w, *,
                                  workspace: Optional[torch.Tensor] = None, stream=None):
    """dvp_fused_lmhead_rows with the number of rows[] entries in use read on the device (n_sub: int32 [1])."""
    n, d = hidden.shape
    v = w_train.shape[0]
    p = DvpLmHeadParams(n, d, v, hidden.stride(0), w_train.stride(0), float(log_rho_value))
    max_rows = rows.numel()
    if workspace is None:
        need = int(lib().dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(p), max_rows))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=hidden.device)
    st = lib().dvp_fused_lmhead_rows_counted(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(ids), _ptr(grad_out),
                                             _ptr(rows), _ptr(n_sub), max_rows, _ptr(d_hidden), _ptr(d_w), _ptr(workspace),
                                             workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_rows_counted")


class LmHeadSaved:
    """What dvp_fused_lmhead_forward leaves for dvp_fused_lmhead_backward."""

    def __init__(self, params, saved, workspace, hidden, w_train, ids):
        self.params, self.saved, self.workspace = params, saved, workspace
        self.hidden, self.w_train, self.ids = hidden, w_train, ids


def dvp_fused_lmhead_forward(hidden, w_train, w_infer, ids, log_rho_value, *, lse_full=False, infer_f8=None,
                             saved: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                             stream=None):
    """Forward of both sides; keeps what the backward needs.  Returns (LmHeadResult without gradients, LmHeadSaved)."""
    for name, t in (("hidden", hidden), ("w_train", w_train)):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 2 or t.stride(1) != 1:
            raise ValueError("%s must be a bf16 [rows, d] GPU tensor with unit inner stride" % name)
    n, d = hidden.shape
    v = w_train.shape[0]
    dev = hidden.device
    p = DvpLmHeadParams(n, d, v, hidden.stride(0), w_train.stride(0), float(log_rho_value))
    if workspace is None:
        workspace = torch.empty(max(int(lib().dvp_fused_lmhead_workspace_bytes(ctypes.byref(p))), 256),
                                dtype=torch.uint8, device=dev)
    if saved is None:
        saved = torch.empty(max(int(lib().dvp_fused_lmhead_saved_bytes(ctypes.byref(p))), 256), dtype=torch.uint8,
                            device=dev)
    out_train = SideOutputs(n, v, dev, lse_full, False)
    has_infer = w_infer is not None or infer_f8 is not None
    out_infer = SideOutputs(n, v, dev, lse_full, False) if has_infer else None
    row_flags = torch.empty(n, dtype=torch.uint8, device=dev)
    side = None
    if infer_f8 is not None:
        h8, w8, scale = infer_f8
        side = ctypes.byref(DvpLmHeadF8Side(h8.data_ptr(), w8.data_ptr(), h8.stride(0), w8.stride(0), float(scale)))
    st = lib().dvp_fused_lmhead_forward(ctypes.byref(p), _ptr(hidden), _ptr(w_train), _ptr(w_infer), side, _ptr(ids),
                                        ctypes.byref(out_train.struct()),
                                        ctypes.byref(out_infer.struct()) if out_infer is not None else None,
                                        _ptr(row_flags), _ptr(saved), saved.numel(), _ptr(workspace),
                                        workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_forward")
    return (LmHeadResult(out_train, out_infer, row_flags, None, None),
            LmHeadSaved(p, saved, workspace, hidden, w_train, ids))


def dvp_fused_lmhead_backward(kept: LmHeadSaved, grad_out, *, d_hidden=None, d_w=None, stream=None):
    """dH, dW from what the forward kept and the now known grad_out."""
    p = kept.params
    dev = kept.hidden.device
    if d_hidden is None:
        d_hidden = torch.empty(p.n_rows, p.ld_hidden, dtype=torch.float32, device=dev)[:, :p.hidden]
    if d_w is None:
        d_w = torch.empty(p.vocab, p.ld_w, dtype=torch.float32, device=dev)[:, :p.hidden]
    st = lib().dvp_fused_lmhead_backward(ctypes.byref(p), _ptr(kept.hidden), _ptr(kept.w_train), _ptr(kept.ids),
                                         _ptr(grad_out), _ptr(kept.saved), kept.saved.numel(), _ptr(d_hidden),
                                         _ptr(d_w), _ptr(kept.workspace), kept.workspace.numel(), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_fused_lmhead_backward")
    return d_hidden, d_w


class SequenceResult:
    def __init__(self, weight, seq_log_ratio, seq_min_weight, seq_veto):
        self.weight, self.seq_log_ratio = weight, seq_log_ratio
        self.seq_min_weight, self.seq_veto = seq_min_weight, seq_veto


def log_threshold(threshold: float) -> float:
    """(float)log(threshold) as the library computes it (token veto, 1e-4 in the paper)."""
    return float(lib().dvp_log_threshold(float(threshold)))


def dvp_sequence_weights(logp_train, logp_infer, seq_offsets, log_threshold_value, *, weight=None,
                         seq_log_ratio=None, seq_min_weight=None, seq_veto=None,
                         stream=None) -> SequenceResult:
    for name, t in (("logp_train", logp_train), ("logp_infer", logp_infer)):
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 1 or not t.is_contiguous():
            raise ValueError("%s must be a contiguous float32 [N] GPU tensor" % name)
    if not seq_offsets.is_cuda or seq_offsets.dtype != torch.int64 or seq_offsets.dim() != 1:
        raise ValueError("seq_offsets must be an int64 [n_seq + 1] GPU tensor")
    n, n_seq = logp_train.shape[0], seq_offsets.shape[0] - 1
    dev = logp_train.device
    if weight is None:
        weight = torch.empty(n, dtype=torch.float32, device=dev)
    if seq_log_ratio is None:
        seq_log_ratio = torch.empty(n_seq, dtype=torch.float32, device=dev)
    if seq_min_weight is None:
        seq_min_weight = torch.empty(n_seq, dtype=torch.float32, device=dev)
    if seq_veto is None:
        seq_veto = torch.empty(n_seq, dtype=torch.uint8, device=dev)
    st = lib().dvp_sequence_weights(n, n_seq, _ptr(logp_train), _ptr(logp_infer), _ptr(seq_offsets),
                                    float(log_threshold_value), _ptr(weight), _ptr(seq_log_ratio),
                                    _ptr(seq_min_weight), _ptr(seq_veto), _stream(stream))
    if st != 0:
        raise DvpError(st, "dvp_sequence_weights")
    return SequenceResult(weight, seq_log_ratio, seq_min_weight, seq_veto)
