"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol that
include/ocs.h declares, and rejects bad arguments before any device work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import ref
from paper_1901_09504_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ocs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ocs_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"ocs_num_splits", "ocs_split_weights", "ocs_quantize", "ocs_split_act", "ocs_qgemm",
            "ocs_select_channels", "ocs_workspace_bytes", "ocs_strerror"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
        assert hasattr(B, n) or n in ("ocs_strerror", "ocs_last_hip_error"), f"binding lacks {n}"


def test_num_splits_matches_oracle_everywhere():
    for Cn in list(range(1, 300)) + [512, 1000, 1024, 1500, 2048, 3000, 4096]:
        for r in (0.0, 0.01, 0.02, 0.05, 0.1, 0.2, 0.25, 0.5, 1.0):
            assert B.ocs_num_splits(Cn, r) == ref.num_splits(Cn, r), (Cn, r)
    assert B.ocs_num_splits(0, 0.1) == 0 and B.ocs_num_splits(10, -1.0) == 0


def test_padded_cols_and_workspace():
    assert B.ocs_padded_cols(2358) == 2432
    assert B.ocs_conv_weight_cols(9, 272) == 2496 and B.ocs_conv_weight_cols(0, 16) == 0
    assert B.ocs_padded_channels(262) == 272 and B.ocs_padded_channels(4) == 16
    assert B.ocs_padded_cols(64) == 64 and B.ocs_padded_cols(269) == 272 and B.ocs_padded_cols(68) == 80 and B.ocs_padded_cols(320) == 320 and B.ocs_padded_cols(321) == 384 and B.ocs_padded_cols(0) == 0
    assert B.ocs_workspace_bytes(0, 10) == 0
    for rows, cols in [(1, 1), (64, 256), (12544, 2304), (6000, 3000), (3211264, 147), (802816, 64)]:
        wb = B.ocs_workspace_bytes(rows, cols)
        assert wb >= 4 * cols and wb % 256 == 0
        assert wb < 64 << 20


A = 1 << 20  # a fake, suitably aligned "device address": validation never dereferences it


def _call(fn, *args):
    return getattr(B.lib(), fn)(*args)


def test_argument_errors_are_reported_without_a_device():
    L = B.lib()
    ws = 1 << 24
    # NULL pointers
    assert L.ocs_quantize(None, 4, 4, 4, 8, None, 1.0, A, 64, A, A, ws, None) == -1
    assert L.ocs_split_act(A, 4, 4, 1, 4, None, None, 2, 8, None, 1.0, A, 64, A, A, ws, None) == -1
    assert L.ocs_split_weights(A, 4, 4, 1, 4, 1, 0, None, A, A, None, 0, None, 8, 1.0, None, 0, None, A, ws, None) == -1
    assert L.ocs_split_weights(A, 4, 4, 1, 4, 1, 0, A, A, A, None, 0, None, 8, 1.0, A, 64, None, A, ws, None) == -1
    assert L.ocs_qgemm(A, 64, A, 64, 4, 4, 4, 8, 8, A, A, None, 0, None, 4, None, 0, None) == -1
    assert L.ocs_split_weights_qa(A, 4, 4, 1, 4, 1, A, A, A, None, A, 8, 8, 1.0, A, 64, A, A, ws, None) == -1  # no chan_path
    assert L.ocs_split_weights_qa(A, 4, 4, 1, 4, 1, A, A, A, A, None, 0, 8, 1.0, None, 0, A, A, ws, None) == -1  # no output
    assert L.ocs_split_weights_qa(A, 4, 4, 1, 4, 1, A, A, A, A, A, 4, 8, 1.0, None, 0, A, A, ws, None) == -2    # ldo < (C+s)*g
    assert L.ocs_split_weights_qa(A, 4, 4, 1, 4, 1, A, A, A, A, A, 8, 9, 1.0, None, 0, A, A, ws, None) == -4    # bits
    assert L.ocs_mse_clip_threshold(A, 4, 4, 4, 8, 16, 4, A, None, A, A, ws, None) == -1   # no histogram
    assert L.ocs_mse_clip_threshold(A, 4, 4, 4, 8, 16, 4, A, A, None, A, ws, None) == -1   # no error array
    assert L.ocs_mse_clip_threshold(A, 4, 4, 4, 8, 0, 4, A, A, A, A, ws, None) == -2       # no bins
    assert L.ocs_mse_clip_threshold(A, 4, 4, 4, 8, 9000, 4, A, A, A, A, ws, None) == -2
    assert L.ocs_mse_clip_threshold(A, 4, 4, 4, 1, 16, 4, A, A, A, A, ws, None) == -4
    assert L.ocs_qconv(A, 64, 1, 4, 4, 8, 3, 3, 1, 1, None, 4, 8, 8, A, A, None, 0, A, 4, None) == -1      # no weights
    assert L.ocs_qconv(A, 64, 1, 2, 2, 8, 3, 3, 1, 0, A, 4, 8, 8, A, A, None, 0, A, 4, None) == -2         # kernel larger than image
    assert L.ocs_qconv(A, 72, 1, 4, 4, 8, 3, 3, 1, 1, A, 4, 8, 8, A, A, None, 0, A, 4, None) == -3         # ldc % 16
    assert L.ocs_qconv(A, 64, 1, 4, 4, 80, 3, 3, 1, 1, A, 4, 8, 8, A, A, None, 0, A, 4, None) == -2        # ldc < C_exp
    assert L.ocs_conv_weights_tap_major(A, 4, 8, 9, 64, A, 64, None) == -2                                  # ldq < C_exp*g
    assert L.ocs_qgemm_requant(A, 64, A, 64, 4, 4, 4, 8, 8, A, A, 0, None, 8, None, 0, A, 16, None, None, 0, None) == -1   # no grid
    assert L.ocs_qgemm_requant(A, 64, A, 64, 4, 4, 4, 8, 8, A, A, 0, A, 8, None, 2, A, 16, None, None, 0, None) == -1      # no list
    assert L.ocs_qgemm_requant(A, 64, A, 64, 4, 20, 4, 8, 8, A, A, 0, A, 8, None, 0, A, 16, None, None, 0, None) == -2     # ldyq < N
    assert L.ocs_qgemm_requant(A, 64, A, 64, 4, 4, 4, 8, 8, A, A, 0, A, 8, None, 0, A, 24, None, None, 0, None) == -3      # ldyq % 16
    assert L.ocs_qgemm_requant(A, 64, A, 64, 4, 4, 4, 8, 8, A, A, 0, A, 8, None, 0, A, 16, A, None, 0, None) == -9         # scale_out aliases the grid
    assert L.ocs_fold_weights(A, 64, 4, 4, 1, 2, None, A, 64, A, None) == -1          # split list missing
    assert L.ocs_fold_weights(A, 4, 4, 4, 1, 2, A, A, 64, A, None) == -2             # ldq < (C+s)*g
    assert L.ocs_split_act_qa(A, 4, 4, 1, 4, A, A, A, A, 1, 8, None, A, 64, A, None) == -1     # no threshold
    assert L.ocs_split_act_qa(A, 4, 4, 1, 4, A, A, A, A, 1, 8, A, A, 64, A, None) == -9        # scale_out aliases it
    # shapes
    assert L.ocs_quantize(A, 0, 4, 4, 8, A, 1.0, A, 64, A, A, ws, None) == -2
    assert L.ocs_quantize(A, 4, 8, 4, 8, A, 1.0, A, 64, A, A, ws, None) == -2      # ldx < cols
    assert L.ocs_quantize(A, 4, 100, 100, 8, A, 1.0, A, 64, A, A, ws, None) == -2   # ldq < cols
    assert L.ocs_split_act(A, 4, 4, 0, 4, A, None, 0, 8, A, 1.0, A, 64, A, A, ws, None) == -2
    assert L.ocs_qgemm(A, 64, A, 64, 4, 4, 100, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -2  # ld < Kpad
    assert L.ocs_qgemm(A, 64, A, 64, 4, 8, 4, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -2    # ldy < N
    # a short K: the pitch only has to hold the row in 16-byte pieces; a long K: whole K-steps
    assert L.ocs_qgemm(A, 64, A, 80, 4, 4, 68, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -2   # 64 < 68
    assert L.ocs_qgemm(A, 88, A, 80, 4, 4, 68, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -3   # 88 % 16
    assert L.ocs_qgemm(A, 400, A, 448, 4, 4, 390, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -2  # 400 < 448
    assert L.ocs_qgemm(A, 464, A, 448, 4, 4, 390, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -3  # 464 % 64
    # alignment
    assert L.ocs_quantize(A, 4, 4, 4, 8, A, 1.0, A, 40, A, A, ws, None) == -3
    assert L.ocs_quantize(A, 4, 4, 4, 8, A, 1.0, A + 4, 64, A, A, ws, None) == -3
    assert L.ocs_qgemm(A + 1, 64, A, 64, 4, 4, 4, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -3
    assert L.ocs_quantize(A, 4, 4, 4, 8, None, 1.0, A, 64, A, A + 16, ws, None) == -3   # workspace
    # bits
    for bits in (1, 9, 0, -3):
        assert L.ocs_quantize(A, 4, 4, 4, bits, A, 1.0, A, 64, A, A, ws, None) == -4
    assert L.ocs_qgemm(A, 64, A, 64, 4, 4, 4, 8, 9, A, A, None, 0, A, 4, None, 0, None) == -4
    # splits
    assert L.ocs_split_act(A, 4, 4, 1, 4, A, None, -1, 8, A, 1.0, A, 64, A, A, ws, None) == -5
    assert L.ocs_select_channels(A, 4, 7000, 1, 7000, 1001, A, A, A, None, A, ws, None) == -5
    # overflow: 140000 * 127 * 127 >= 2^31, but fine at 4-bit weights
    ld = 140032
    assert L.ocs_qgemm(A, ld, A, ld, 4, 4, 140000, 8, 8, A, A, None, 0, A, 4, None, 0, None) == -6
    # workspace
    assert L.ocs_quantize(A, 4, 4, 4, 8, None, 1.0, A, 64, A, None, 0, None) == -7
    assert L.ocs_quantize(A, 4, 4, 4, 8, None, 1.0, A, 64, A, A, 16, None) == -7
    assert L.ocs_select_channels(A, 12544, 256, 9, 2304, 6, A, A, A, None, A, 1024, None) == -7
    # mode / key
    assert L.ocs_split_weights(A, 4, 4, 1, 4, 1, 7, A, A, A, None, 0, None, 8, 1.0, None, 0, None, A, ws, None) == -9
    assert L.ocs_tune(b"no_such_key", 1) == -9
    # clip ratio
    for bad in (0.0, -0.5, float("nan"), float("inf")):
        assert L.ocs_quantize(A, 4, 4, 4, 8, None, bad, A, 64, A, A, ws, None) == -10
        assert L.ocs_split_act(A, 4, 4, 1, 4, A, None, 1, 8, None, bad, A, 64, A, A, ws, None) == -10
        assert L.ocs_act_threshold(A, 4, 4, 1, 4, A, None, 1, 8, bad, A, A, ws, None) == -10
        assert L.ocs_split_weights(A, 4, 4, 1, 4, 1, 0, A, A, A, None, 0, None, 8, bad, A, 64, A, A, ws, None) == -10
        assert L.ocs_split_weights_qa(A, 4, 4, 1, 4, 1, A, A, A, A, A, 8, 8, bad, None, 0, A, A, ws, None) == -10
    assert L.ocs_quantize(A, 0, 4, 4, 8, A, -1.0, A, 64, A, A, ws, None) == -2   # a given threshold: the ratio is unused
    for code in range(-10, 1):
        assert len(L.ocs_strerror(code)) > 1
    assert L.ocs_strerror(-99) == b"unknown error code"


def test_static_scratch_entry_point_checks_arguments_and_size_on_the_host():
    L = B.lib()
    # the same argument checks as ocs_split_act, in the same order
    assert L.ocs_split_act_static(None, 4, 4, 1, 4, None, None, 0, 8, None, 1.0, A, 64, A, None) == -1
    assert L.ocs_split_act_static(A, 4, 4, 0, 4, A, None, 0, 8, A, 1.0, A, 64, A, None) == -2
    assert L.ocs_split_act_static(A, 4, 4, 1, 4, A, None, -1, 8, A, 1.0, A, 64, A, None) == -5
    assert L.ocs_split_act_static(A, 4, 4, 1, 4, A, None, 1, 9, A, 1.0, A, 64, A, None) == -4
    assert L.ocs_split_act_static(A, 4, 4, 1, 4, A, None, 1, 8, None, 0.0, A, 64, A, None) == -10
    # a tensor whose scratch need is beyond the array: refused before any device work
    M, Cn, g = 64, 4000, 256                      # the column maxima alone are 4 MB
    assert B.ocs_workspace_bytes(M, Cn * g) > B.STATIC_SCRATCH_BYTES
    assert L.ocs_split_act_static(A, M, Cn, g, Cn * g, None, None, 0, 8, None, 1.0, A, Cn * g, A, None) == -7
    assert L.ocs_split_act_static(A, M, Cn, g, Cn * g, None, None, 0, 8, A, 1.0, A, Cn * g, A, None) == -7
    # every layer shape of the five workloads fits
    from paper_1901_09504_amd import workloads as wl
    for cfg in range(1, 6):
        for layer in wl.config(cfg):
            assert B.ocs_workspace_bytes(layer.M, layer.C * layer.g) <= B.STATIC_SCRATCH_BYTES, layer


def test_split_k_entry_point_checks_shape_and_workspace_on_the_host():
    L = B.lib()
    args = lambda M, N, K, parts, ws, wb: (A, 4864, A, 4864, M, N, K, 8, 8, A, A, None, 0, A, N, parts, ws, wb, None)
    assert B.ocs_qgemm_split_k_workspace_bytes(12544, 512, 4842, 2) == 49 * 2 * 2 * 256 * 256 * 4
    assert B.ocs_qgemm_split_k_workspace_bytes(12544, 512, 4842, 1) == 0        # nothing to split
    assert B.ocs_qgemm_split_k_workspace_bytes(50176, 512, 4842, 2) == 0        # 392 tiles: no counter slot that large
    assert B.ocs_qgemm_split_k_workspace_bytes(256, 256, 128, 3) == 0           # two K-steps, three parts
    assert L.ocs_qgemm_split_k(*args(12544, 512, 4842, 1, A, 1 << 30)) == -2
    assert L.ocs_qgemm_split_k(*args(50176, 512, 4842, 2, A, 1 << 30)) == -2
    assert L.ocs_qgemm_split_k(*args(12544, 512, 4842, 2, None, 0)) == -7
    assert L.ocs_qgemm_split_k(*args(12544, 512, 4842, 2, A, 1000)) == -7
    assert L.ocs_qgemm_split_k(*args(12544, 512, 4842, 2, A + 8, 1 << 30)) == -3
    # the split walks whole K-steps: the tight pitch ocs_qgemm takes for a short K is refused
    short = lambda ld: (A, ld, A, ld, 256, 256, 269, 8, 8, A, A, None, 0, A, 256, 2, A, 1 << 30, None)
    assert L.ocs_qgemm_split_k(*short(272)) == -2
    assert L.ocs_qgemm_split_k(*short(336)) == -3


def test_one_launch_entry_point_says_what_it_serves_and_checks_on_the_host():
    L = B.lib()
    assert B.ocs_split_act_qgemm_fits(802816, 64, 9, 4, 64, 576) and B.ocs_split_act_qgemm_pays(802816, 64, 9, 4, 64, 576)
    assert B.ocs_split_act_qgemm_fits(802816, 64, 1, 4, 256, 64) and not B.ocs_split_act_qgemm_pays(802816, 64, 1, 4, 256, 64)
    assert B.ocs_split_act_qgemm_fits(3211264, 3, 49, 1, 64, 147)          # 147 columns: two whole K-steps and a rest
    assert not B.ocs_split_act_qgemm_fits(100, 3, 9, 1, 64, 27)            # less than one K-step
    assert not B.ocs_split_act_qgemm_fits(12544, 512, 9, 26, 512, 4608)    # more than one tile of output columns
    assert not B.ocs_split_act_qgemm_fits(100, 64, 256, 4, 64, 16384)      # 16384 columns
    assert not B.ocs_split_act_qgemm_fits(100, 64, 64, 40, 64, 4096)       # 2560 appended columns
    call = lambda **k: L.ocs_split_act_qgemm(*[k.get(n, d) for n, d in (
        ("X", A), ("M", 128), ("C", 64), ("g", 1), ("ldx", 64), ("cs", A), ("s", 4), ("bx", 8), ("thr", A), ("Wq", A),
        ("ldw", 80), ("N", 64), ("bw", 8), ("sw", A), ("sxo", None), ("acc", None), ("ldacc", 0), ("Y", A), ("ldy", 64),
        ("stream", None))])
    assert call(X=None) == -1 and call(thr=None) == -1 and call(Wq=None) == -1 and call(Y=None) == -1 and call(cs=None) == -1
    assert call(ldx=60) == -2 and call(ldy=63) == -2 and call(ldw=64) == -2 and call(acc=A, ldacc=8) == -2
    assert call(N=300, ldy=300) == -2 and call(C=3, g=9, ldx=27, s=1, ldw=48) == -2     # not served
    assert call(ldw=88) == -3 and call(Wq=A + 4) == -3
    assert call(bx=9) == -4 and call(s=-1) == -5
    assert call(sxo=A, thr=A) == -9


def test_binding_raises_on_error():
    with pytest.raises(B.OcsError) as e:
        B._check(-4, "ocs_quantize")
    assert "2..8" in str(e.value) and e.value.code == -4
