"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import math
import re
from pathlib import Path

import pytest

from paper_2512_23087_amd import dvp

ROOT = Path(__file__).resolve().parents[1]
FAKE = 0x10000   # never dereferenced: every call below fails validation or has zero rows


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "dvp.h").read_text()
    declared = set(re.findall(r"\b(dvp_[a-z_0-9]+)\s*\(", header))
    assert declared == set(dvp.EXPORTS)
    L = dvp.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_log_rho_and_status_strings():
    assert dvp.log_rho(math.exp(-13.0)) == -13.0
    assert dvp.log_rho(1.0) == 0.0
    assert dvp.log_rho(0.0) == -math.inf
    assert math.isnan(dvp.log_rho(2.0)) and math.isnan(dvp.log_rho(-1.0))
    assert dvp.status_string(0) == "ok"
    texts = {dvp.status_string(i) for i in range(9)}
    assert len(texts) == 9 and dvp.status_string(99) == "unknown status"


def _fwd(p, z_train=FAKE, z_infer=FAKE, ids=FAKE, out_train=True, out_infer=True):
    so = dvp.DvpSideOut(FAKE, FAKE, FAKE, None, FAKE, None)
    return dvp.lib().dvp_forward(ctypes.byref(p), z_train, z_infer, ids,
                                 ctypes.byref(so) if out_train else None,
                                 ctypes.byref(so) if out_infer else None, FAKE, None)


def test_argument_validation_needs_no_gpu():
    ok = dict(n_rows=0, vocab=100, ld_train=100, ld_infer=100, ld_grad=100, dtype=1, log_rho=-3.0)

    def P(**kw):
        d = dict(ok); d.update(kw)
        return dvp.DvpParams(d["n_rows"], d["vocab"], d["ld_train"], d["ld_infer"], d["ld_grad"],
                             d["dtype"], d["log_rho"], d.get("dtype_infer", d["dtype"]), d.get("mode", 0),
                             d.get("mask_value", 0.0))

    assert _fwd(P()) == 0                                   # zero rows: nothing to do
    assert _fwd(P(), z_train=None, ids=None) == 0           # ... and no pointer is looked at
    assert dvp.lib().dvp_forward(None, FAKE, FAKE, FAKE, None, None, None, None) == 1
    assert _fwd(P(n_rows=1), z_train=None) == 1
    assert _fwd(P(n_rows=1), ids=None) == 1
    assert _fwd(P(n_rows=1), out_train=False) == 1
    assert _fwd(P(vocab=0)) == 2
    assert _fwd(P(n_rows=-1)) == 2
    assert _fwd(P(ld_train=99)) == 2
    assert _fwd(P(ld_infer=99)) == 2
    assert _fwd(P(ld_infer=99), z_infer=None) == 0          # ignored without an inference side
    assert _fwd(P(vocab=2 ** 31 - 2 ** 16 + 1, ld_train=2 ** 31, ld_infer=2 ** 31)) == 2
    assert _fwd(P(vocab=2 ** 31 - 2 ** 16, ld_train=2 ** 31, ld_infer=2 ** 31)) == 0
    assert _fwd(P(dtype=7)) == 3
    assert _fwd(P(mode=1, mask_value=-50.0)) == 0 and _fwd(P(mode=2)) == 3
    assert _fwd(P(mode=1, mask_value=float("nan"))) == 3 and _fwd(P(mode=1, mask_value=-math.inf)) == 3
    assert _fwd(P(mode=1, mask_value=-50.0, dtype_infer=2)) == 3   # no storage arithmetic to round the threshold in
    assert _fwd(P(mode=0, mask_value=float("nan"))) == 0          # ignored by the exact rule
    assert _fwd(P(dtype=2)) == 3                            # 8-bit logits are an inference-side format only
    assert _fwd(P(dtype=1, dtype_infer=0)) == 3             # the two sides differ only by the 8-bit case
    assert _fwd(P(dtype=1, dtype_infer=2)) == 0 and _fwd(P(dtype=0, dtype_infer=2)) == 0
    assert _fwd(P(dtype=1, dtype_infer=9), z_infer=None) == 0   # ignored without an inference side
    assert _fwd(P(n_rows=1, dtype=1, dtype_infer=2), z_infer=FAKE + 1) != 4   # bytes need no alignment
    assert _fwd(P(log_rho=0.5)) == 3
    assert _fwd(P(log_rho=float("nan"))) == 3
    assert _fwd(P(log_rho=-math.inf)) == 0
    assert _fwd(P(n_rows=1), z_train=FAKE + 1) == 4         # not aligned to the element size
    assert _fwd(P(n_rows=1, dtype=0), z_infer=FAKE + 2) == 4

    L = dvp.lib()
    so = dvp.DvpSideOut(FAKE, FAKE, FAKE, None, FAKE, None)
    p = P()
    p1 = P(n_rows=1)
    assert L.dvp_forward_backward(ctypes.byref(p1), FAKE, FAKE, FAKE, None, ctypes.byref(so),
                                  ctypes.byref(so), FAKE, FAKE, None) == 1     # grad_out missing
    assert L.dvp_forward_backward(ctypes.byref(P(ld_grad=5)), FAKE, FAKE, FAKE, FAKE,
                                  ctypes.byref(so), ctypes.byref(so), FAKE, FAKE, None) == 2
    assert L.dvp_backward(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == 0
    assert L.dvp_backward(ctypes.byref(p1), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None) == 1
    assert L.dvp_backward(ctypes.byref(p1), FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, None) == 1


def test_row_path_selection():
    L = dvp.lib()

    def path(v, dtype, ld=None, aligned=1, dtype_infer=None):
        p = dvp.DvpParams(4, v, ld or v, ld or v, ld or v, dtype, -1.0, dtype if dtype_infer is None else dtype_infer)
        return L.dvp_row_path(ctypes.byref(p), aligned)

    assert path(151936, 1) == 1 and path(32000, 1) == 1 and path(32000, 0) == 1
    assert path(163840, 1) == 1 and path(163848, 1) == 1       # beyond the register file: partly re-read, same kernel
    assert path(81920, 0) == 1 and path(81924, 0) == 1 and path(151936, 0) == 1
    assert path(163848, 1, dtype_infer=2) == 0                 # byte inference rows: only while the bf16 row fits
    assert path(1000, 1, ld=1001) == 0                         # rows not 16-byte aligned
    assert path(1000, 1, aligned=0) == 0
    assert path(7, 1) == 0 and path(8, 1, ld=8) == 1               # shorter than one vector
    assert path(3, 0) == 0 and path(4, 0) == 1
    assert path(0, 1) == -1
    p = dvp.DvpParams(4, 32000, 32000, 32000, 32000, 1, -1.0, 1, 1, -50.0)
    assert L.dvp_row_path(ctypes.byref(p), 1) == 0                # the finite-mask variant is re-read
    # 8-bit inference rows: single-read next to bf16 training rows of at least one 16-token vector
    assert path(151936, 1, dtype_infer=2) == 1 and path(32000, 1, dtype_infer=2) == 1
    assert path(32008, 1, dtype_infer=2) == 0                  # 32008 bytes per inference row: not 16-byte aligned
    assert path(8, 1, dtype_infer=2) == 0 and path(16, 1, dtype_infer=2) == 1
    assert path(32000, 0, dtype_infer=2) == 0                  # fp32 training rows take the re-reading path


def test_binding_refuses_cpu_tensors():
    import torch
    z = torch.zeros(2, 8, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        dvp.dvp_forward(z, None, torch.zeros(2, dtype=torch.int64), -1.0)


def test_sequence_weights_validation_needs_no_gpu():
    L = dvp.lib()

    def call(n_tokens=8, n_seq=0, lt=FAKE, li=FAKE, off=FAKE, lthr=-9.0, w=FAKE, r=FAKE, mn=FAKE, v=FAKE):
        return L.dvp_sequence_weights(n_tokens, n_seq, lt, li, off, lthr, w, r, mn, v, None)

    assert call() == 0 and call(lt=None, off=None) == 0       # zero sequences: nothing to do
    assert call(n_seq=-1) == 2 and call(n_tokens=-1) == 2
    assert call(lthr=float("nan")) == 3
    assert call(n_seq=1, lt=None) == 1 and call(n_seq=1, off=None) == 1 and call(n_seq=1, v=None) == 1
    assert call(n_seq=1, r=None) == 1
    assert call(n_seq=1, off=FAKE + 4) == 4 and call(n_seq=1, w=FAKE + 2) == 4
    assert dvp.log_threshold(1e-4) == pytest.approx(math.log(1e-4), rel=1e-7)
    assert math.isnan(dvp.log_threshold(0.0)) and math.isnan(dvp.log_threshold(-1.0))


def test_sparse_gradient_validation_needs_no_gpu():
    L = dvp.lib()
    so = dvp.DvpSideOut(FAKE, FAKE, FAKE, None, FAKE, None)

    def call(n_rows=1, vocab=32000, cap=64, z=FAKE, flags=FAKE, entries=FAKE, dtype=1, ld=None):
        p = dvp.DvpParams(n_rows, vocab, ld or vocab, ld or vocab, 0, dtype, -3.0, dtype)
        return L.dvp_forward_backward_sparse(ctypes.byref(p), z, FAKE, FAKE, FAKE, ctypes.byref(so),
                                             ctypes.byref(so), flags, entries, FAKE, cap, None)

    assert call(n_rows=0) == 0
    assert call(cap=0) == 3 and call(cap=65537) == 3
    assert call(flags=None) == 1 and call(entries=None) == 1 and call(z=None) == 1
    assert call(entries=FAKE + 4) == 4
    assert call(vocab=32001) == 5            # rows not 16-byte aligned: no single-read path
    assert call(z=FAKE + 2) == 5             # base pointer not 16-byte aligned


def test_lists_to_dense_validation_needs_no_gpu():
    L = dvp.lib()

    def call(n_rows=1, vocab=32000, cap=64, entries=FAKE, glen=FAKE, flags=FAKE, grad=FAKE, z=None, ids=None,
             m=None, lse=None, dz=FAKE, ld_grad=None, mode=0):
        p = dvp.DvpParams(n_rows, vocab, vocab, 0, vocab if ld_grad is None else ld_grad, 1, -3.0, 1, mode, -50.0)
        return L.dvp_lists_to_dense(ctypes.byref(p), entries, glen, cap, flags, grad, z, ids, m, lse, dz, None)

    assert call(n_rows=0) == 0
    assert call(cap=0) == 3 and call(mode=1) == 5
    assert call(entries=None) == 1 and call(glen=None) == 1 and call(flags=None) == 1 and call(dz=None) == 1
    assert call(z=FAKE) == 1 and call(z=FAKE, ids=FAKE, m=FAKE, lse=FAKE, grad=None) == 1
    assert call(ld_grad=31999) == 2
    assert call(entries=FAKE + 4) == 4 and call(dz=FAKE + 1) == 4


def test_lmhead_argument_validation_needs_no_gpu():
    L = dvp.lib()
    so = dvp.DvpSideOut(FAKE, FAKE, FAKE, None, FAKE, None)
    ws = FAKE * 256

    def P(n=1, d=128, v=64, ld_h=None, ld_w=None, lr=-3.0):
        return dvp.DvpLmHeadParams(n, d, v, ld_h or d, ld_w or d, lr)

    def call(p, hidden=FAKE, w=FAKE, w_infer=FAKE, ids=FAKE, grad=None, bytes_=1 << 40, workspace=ws):
        return L.dvp_fused_lmhead(ctypes.byref(p), hidden, w, w_infer, ids, grad, ctypes.byref(so), ctypes.byref(so),
                                  FAKE, None, None, workspace, bytes_, None)

    assert L.dvp_fused_lmhead_workspace_bytes(ctypes.byref(P())) > 0
    assert L.dvp_fused_lmhead_workspace_bytes(ctypes.byref(P(d=100))) == 0
    assert call(P(n=0)) == 0
    assert call(P(), hidden=None) == 1
    assert call(P(lr=0.5)) == 3
    assert call(P(v=0)) == 2
    assert call(P(d=96)) == 5                       # hidden size not a multiple of 64
    assert call(P(v=(1 << 22) + 1)) == 5
    assert call(P(), grad=FAKE) == 1                # gradient outputs missing
    assert call(P(), hidden=FAKE + 8) == 4
    assert call(P(), bytes_=16) == 6 and call(P(), workspace=None) == 6

    # forward and backward as two calls
    # the masked exponentials of 300 rows x 1000 tokens as bf16, padded to whole 256 x 256 tiles, and two factors per row
    saved_bytes = L.dvp_fused_lmhead_saved_bytes(ctypes.byref(P(n=300, v=1000)))
    assert 512 * 1024 * 2 + 2 * 300 * 4 <= saved_bytes <= 512 * 1024 * 2 + 2 * 300 * 4 + 1024
    assert L.dvp_fused_lmhead_saved_bytes(ctypes.byref(P(d=100))) == 0

    def fwd(p, saved=ws, saved_bytes=1 << 40, w_infer=FAKE, side=None):
        return L.dvp_fused_lmhead_forward(ctypes.byref(p), FAKE, FAKE, w_infer, side, FAKE, ctypes.byref(so),
                                          ctypes.byref(so), FAKE, saved, saved_bytes, ws, 1 << 40, None)

    def bwd(p, grad=FAKE, saved=ws, saved_bytes=1 << 40, dh=FAKE, dw=FAKE):
        return L.dvp_fused_lmhead_backward(ctypes.byref(p), FAKE, FAKE, FAKE, grad, saved, saved_bytes, dh, dw, ws,
                                           1 << 40, None)

    assert fwd(P(n=0)) == 0 and bwd(P(n=0)) == 0
    assert fwd(P(), saved=None) == 6 and fwd(P(), saved_bytes=100) == 6 and fwd(P(), saved=FAKE + 16) == 6
    assert bwd(P(), grad=None) == 1 and bwd(P(), dh=None) == 1 and bwd(P(), saved_bytes=100) == 6
    assert fwd(P(d=96)) == 5 and bwd(P(lr=0.5)) == 3

    def call8(p, side, hidden=FAKE):
        return L.dvp_fused_lmhead_f8infer(ctypes.byref(p), hidden, FAKE, side, FAKE, None, ctypes.byref(so),
                                          ctypes.byref(so), FAKE, None, None, ws, 1 << 40, None)

    def S(hidden=FAKE, w=FAKE, ld_h=128, ld_w=128, scale=0.5):
        return ctypes.byref(dvp.DvpLmHeadF8Side(hidden, w, ld_h, ld_w, scale))

    assert call8(P(), None) == 1
    assert call8(P(), S(hidden=None)) == 1
    assert call8(P(), S(ld_h=64)) == 2              # row stride shorter than the hidden size
    assert call8(P(), S(scale=0.0)) == 3 and call8(P(), S(scale=float("nan"))) == 3
    assert call8(P(d=192, ld_h=192, ld_w=192), S(ld_h=192, ld_w=192)) == 5     # hidden size not a multiple of 128
    assert call8(P(), S(ld_h=136)) == 5             # byte rows not 16-byte aligned
    assert call8(P(), S(w=FAKE + 8)) == 4
    assert call8(P(n=0), S()) == 0
    assert fwd(P(), side=S()) == 3                  # a bf16 and an 8-bit inference side at once
    assert fwd(P(), w_infer=None, side=S(scale=0.0)) == 3

    # gradient as per-row lists
    def lists(p, cap=64, grad=FAKE, flags=FAKE, entries=FAKE, glen=FAKE, dh=FAKE, dw=FAKE, bytes_=1 << 40, side=so):
        return L.dvp_fused_lmhead_lists(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, grad, ctypes.byref(side), ctypes.byref(side),
                                        flags, entries, glen, cap, dh, dw, ws, bytes_, None)

    small = L.dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(P(n=16384, d=4096, v=151936)), 64)
    assert 0 < small < L.dvp_fused_lmhead_workspace_bytes(ctypes.byref(P(n=16384, d=4096, v=151936))) // 4
    assert L.dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(P()), 0) == 0
    assert L.dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(P()), 1025) == 0
    assert L.dvp_fused_lmhead_lists_workspace_bytes(ctypes.byref(P(n=1 << 22)), 1024) == 0     # N * cap >= 2^31
    assert lists(P(n=0)) == 0
    assert lists(P(), cap=0) == 3 and lists(P(), cap=1025) == 5 and lists(P(n=1 << 22), cap=1024) == 5
    assert lists(P(), flags=None) == 1 and lists(P(), entries=None) == 1
    assert lists(P(), grad=None, flags=None, entries=None, glen=None, dh=None, dw=None, bytes_=1000) == 6   # forward only: accepted up to the workspace check
    assert lists(P(), glen=None) == 1 and lists(P(), dh=None) == 1 and lists(P(), dw=None) == 1
    assert lists(P(), entries=FAKE + 4) == 4 and lists(P(), dw=FAKE + 8) == 4
    assert lists(P(), side=dvp.DvpSideOut(FAKE, FAKE, FAKE, None, FAKE, FAKE)) == 5             # no bitmask in this form
    assert lists(P(d=96)) == 5 and lists(P(lr=0.5)) == 3
    assert lists(P(), bytes_=1000) == 6

    def lists8(p, side, cap=64):
        return L.dvp_fused_lmhead_lists_f8infer(ctypes.byref(p), FAKE, FAKE, side, FAKE, FAKE, ctypes.byref(so), ctypes.byref(so),
                                                FAKE, FAKE, FAKE, cap, FAKE, FAKE, ws, 1000, None)

    assert lists8(P(), None) == 1 and lists8(P(), S(hidden=None)) == 1
    assert lists8(P(), S(scale=0.0)) == 3 and lists8(P(), S(ld_h=136)) == 5 and lists8(P(), S(w=FAKE + 8)) == 4
    assert lists8(P(), S()) == 6                    # everything accepted up to the workspace check
    assert lists8(P(n=0), S()) == 0

    # dense gradient of a subset of rows
    def rows_call(p, n_sub=1, rows=FAKE, grad=FAKE, dh=FAKE, dw=FAKE, bytes_=1000):
        return L.dvp_fused_lmhead_rows(ctypes.byref(p), FAKE, FAKE, FAKE, grad, rows, n_sub, dh, dw, ws, bytes_, None)

    assert L.dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(P(n=100)), 10) > 0
    assert L.dvp_fused_lmhead_rows_workspace_bytes(ctypes.byref(P(n=100)), 101) == 0
    assert rows_call(P(n=4), n_sub=0) == 0
    assert rows_call(P(n=4), n_sub=5) == 2 and rows_call(P(n=4), n_sub=-1) == 2
    assert rows_call(P(n=4), rows=None) == 1 and rows_call(P(n=4), grad=None) == 1 and rows_call(P(n=4), dw=None) == 1
    assert rows_call(P(n=4), rows=FAKE + 2) == 4 and rows_call(P(n=4, d=96)) == 5
    assert rows_call(P(n=4)) == 6                   # everything accepted up to the workspace check


C_PROGRAM = r"""
#include <math.h>
#include <stdio.h>
#include <string.h>
#include "dvp.h"

#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    dvp_params p;
    dvp_side_out out;
    dvp_lmhead_params lp;
    memset(&p, 0, sizeof p);
    memset(&out, 0, sizeof out);
    memset(&lp, 0, sizeof lp);

    CHECK(dvp_log_rho(1.0) == 0.0f);
    CHECK(dvp_log_rho(0.0) == -INFINITY);
    CHECK(isnan(dvp_log_rho(1.5)));
    CHECK(fabsf(dvp_log_rho(1e-4) - (float)log(1e-4)) == 0.0f);
    CHECK(fabsf(dvp_log_threshold(1e-4) - (float)log(1e-4)) == 0.0f);
    CHECK(strcmp(dvp_status_string(DVP_OK), "ok") == 0);
    CHECK(strlen(dvp_status_string(DVP_ERR_SCRATCH)) > 0);

    CHECK(dvp_forward(NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == DVP_ERR_NULL);
    p.n_rows = 1; p.vocab = 100; p.ld_train = 100; p.ld_infer = 100; p.ld_grad = 100;
    p.dtype = DVP_BF16; p.dtype_infer = DVP_BF16; p.log_rho = -3.0f; p.mode = DVP_MODE_EXACT;
    CHECK(dvp_forward(&p, NULL, NULL, NULL, &out, NULL, NULL, NULL) == DVP_ERR_NULL);
    p.log_rho = 1.0f;
    CHECK(dvp_forward(&p, NULL, NULL, NULL, &out, NULL, NULL, NULL) == DVP_ERR_PARAM);
    p.log_rho = -3.0f; p.ld_train = 99;
    CHECK(dvp_forward(&p, NULL, NULL, NULL, &out, NULL, NULL, NULL) == DVP_ERR_SHAPE);
    p.ld_train = 100; p.n_rows = 0;
    CHECK(dvp_forward(&p, NULL, NULL, NULL, &out, NULL, NULL, NULL) == DVP_OK);
    CHECK(dvp_backward(&p, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == DVP_OK);
    CHECK(dvp_forward_backward(&p, NULL, NULL, NULL, NULL, &out, NULL, NULL, NULL, NULL) == DVP_OK);
    CHECK(dvp_row_path(&p, 1) == 0);                     /* 200-byte rows: not 16-byte aligned */
    p.vocab = 104; p.ld_train = 104; p.ld_infer = 104; p.ld_grad = 104;
    CHECK(dvp_row_path(&p, 1) == 1);
    CHECK(dvp_row_path(NULL, 1) == -1);

    lp.n_rows = 16; lp.hidden = 128; lp.vocab = 1000; lp.ld_hidden = 128; lp.ld_w = 128; lp.log_rho = -2.0f;
    CHECK(dvp_fused_lmhead_workspace_bytes(&lp) > 0);
    CHECK(dvp_fused_lmhead_workspace_bytes(NULL) == 0);
    CHECK(dvp_fused_lmhead(&lp, NULL, NULL, NULL, NULL, NULL, &out, NULL, NULL, NULL, NULL, NULL, 0, NULL) == DVP_ERR_NULL);
    lp.hidden = 100; lp.ld_hidden = 104; lp.ld_w = 104;
    CHECK(dvp_fused_lmhead(&lp, NULL, NULL, NULL, NULL, NULL, &out, NULL, NULL, NULL, NULL, NULL, 0, NULL) == DVP_ERR_UNSUPPORTED);
    CHECK(dvp_sequence_weights(-1, 1, NULL, NULL, NULL, -9.0f, NULL, NULL, NULL, NULL, NULL) == DVP_ERR_SHAPE);
    CHECK(sizeof(dvp_grad_entry) == 8);
    CHECK(dvp_hbm_probe(9, NULL, NULL, NULL, 1, 16, NULL) == DVP_ERR_PARAM);
    CHECK(dvp_hbm_probe(DVP_PROBE_FILL, NULL, NULL, NULL, 1, 16, NULL) == DVP_ERR_NULL);
    CHECK(dvp_hbm_probe(DVP_PROBE_FILL_WIDE, NULL, NULL, NULL, 1, 24, NULL) == DVP_ERR_SHAPE);
    CHECK(dvp_hbm_probe(DVP_PROBE_READ_ONESHOT, NULL, NULL, NULL, 0, 16, NULL) == DVP_OK);
    CHECK(dvp_set_split_min_bytes(-1) == DVP_SPLIT_MIN_BYTES_DEFAULT);
    CHECK(dvp_set_split_min_bytes(0) == DVP_SPLIT_MIN_BYTES_DEFAULT);
    CHECK(dvp_set_split_min_bytes(DVP_SPLIT_MIN_BYTES_DEFAULT) == 0);
    printf("ok\n");
    return 0;
}
"""


def test_header_is_plain_c11_and_host_entry_points_work_from_c(tmp_path):
    """include/dvp.h compiles as C11 (pedantic, warnings are errors) and a C program linked against the
    library gets the host-only results and the validation codes without a GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    dvp.lib()
    src = tmp_path / "host_check.c"
    src.write_text(C_PROGRAM)
    exe = tmp_path / "host_check"
    libdir = str(dvp.LIB_PATH.parent)
    subprocess.check_call(["gcc", "-std=c11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", str(ROOT / "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-l:libdvp_hip.so", "-lm",
                           "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and res.stdout.strip() == "ok", res.stdout + res.stderr


def test_prepare_is_a_host_call():
    """dvp_prepare touches no data: DVP_OK with a usable GPU, DVP_ERR_HIP without one, never a crash."""
    assert dvp.lib().dvp_prepare() in (0, 7)


def test_split_limit_is_a_process_wide_setting():
    """dvp_set_split_min_bytes: a negative argument reads, anything else sets and returns the value before."""
    assert dvp.set_split_min_bytes(-1) == dvp.SPLIT_MIN_BYTES_DEFAULT
    assert dvp.set_split_min_bytes(12345) == dvp.SPLIT_MIN_BYTES_DEFAULT
    assert dvp.set_split_min_bytes(-7) == 12345
    assert dvp.set_split_min_bytes(dvp.SPLIT_MIN_BYTES_DEFAULT) == 12345
