"""GPU parity, call by call: every entry point of the C ABI against the CPU oracle on the
same seeded inputs.  Integer results (codes, split lists, accumulators) must match bit for
bit; fp32 scales must be identical; dequantized outputs agree within 1e-6 relative."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1901_09504_amd import binding as B

from gpu_util import (assert_y_close, gpu_conv_layer, gpu_mse_clip, gpu_qgemm, gpu_quantize, gpu_select, gpu_split_act,
                      gpu_split_weights, gpu_split_weights_qa, dev, host, require_gpu)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()


def _tensor(rng, rows, cols, kind):
    if kind == "normal":
        x = rng.standard_normal((rows, cols)).astype(np.float32)
    elif kind == "ties":   # multiples of 1/8 up to 16: many exact ties against a power-of-two grid
        x = (rng.integers(-128, 129, (rows, cols)) / 8.0).astype(np.float32)
    elif kind == "heavy":
        x = rng.standard_t(2.0, (rows, cols)).astype(np.float32)
    elif kind == "zero":
        x = np.zeros((rows, cols), dtype=np.float32)
    return x


# ---- ocs_quantize -------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 5), (7, 64), (33, 147), (130, 269), (65, 1000),
                                       (257, 2304), (19, 4099)])
@pytest.mark.parametrize("bits", [2, 5, 8])
@pytest.mark.parametrize("act_map", [0, 1])   # lanes dealt over the output / over the input
def test_quantize_dynamic(rows, cols, bits, act_map):
    rng = np.random.default_rng(rows * 1000 + cols + bits)
    x = _tensor(rng, rows, cols, "heavy")
    q_ref, s_ref = ref.quantize(x, bits, ldq=B.ocs_padded_cols(cols))
    B.ocs_tune("act_map", act_map)
    try:
        q, s = gpu_quantize(x, bits)
    finally:
        B.ocs_tune("act_map", -1)
    assert np.array_equal(s, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("rows,cols", [(1, 1), (1, 3), (3, 5), (7, 65), (33, 147), (130, 269), (257, 1023),
                                       (1031, 1030), (4100, 517)])
@pytest.mark.parametrize("variant", [(0, 256, 1), (1, 256, 1), (1, 256, 4), (1, 1024, 1), (1, 1024, 2), (1, 1024, 4)])
def test_absmax_pass_variants(rows, cols, variant):
    """max|x| of a contiguous tensor: the column pass and every shape of the flat pass give the
    oracle's grid (the largest magnitude sits in the last, partly filled group of four)."""
    flat, bt, un = variant
    rng = np.random.default_rng(rows * 31 + cols)
    x = _tensor(rng, rows, cols, "normal")
    x[-1, -1] = -9.5
    q_ref, s_ref = ref.quantize(x, 8, ldq=B.ocs_padded_cols(cols))
    B.ocs_tune("max_flat", flat); B.ocs_tune("max_bt", bt); B.ocs_tune("max_un", un)
    try:
        q, s = gpu_quantize(x, 8)
    finally:
        B.ocs_tune("max_flat", -1); B.ocs_tune("max_bt", -1); B.ocs_tune("max_un", -1)
    assert np.array_equal(s, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("kind,threshold,clip", [("ties", 16.0, 1.0), ("ties", 15.0, 1.0), ("normal", None, 0.8),
                                                  ("normal", 2.5, 1.0), ("zero", None, 1.0), ("zero", 0.0, 1.0),
                                                  ("heavy", None, 0.3)])
@pytest.mark.parametrize("bits", [3, 4, 6, 7, 8])
def test_quantize_thresholds_and_ties(kind, threshold, clip, bits):
    rng = np.random.default_rng(bits)
    x = _tensor(rng, 61, 333, kind)
    q_ref, s_ref = ref.quantize(x, bits, threshold=threshold, clip_ratio=clip, ldq=B.ocs_padded_cols(333))
    q, s = gpu_quantize(x, bits, threshold=threshold, clip_ratio=clip)
    assert np.array_equal(s, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("ld_extra,misalign", [(0, True), (1, False), (3, True), (4, False)])
def test_quantize_unaligned_inputs(ld_extra, misalign):
    rng = np.random.default_rng(5)
    x = _tensor(rng, 45, 300, "normal")
    q_ref, s_ref = ref.quantize(x, 8, ldq=B.ocs_padded_cols(300))
    q, s = gpu_quantize(x, 8, ld_extra=ld_extra, misalign=misalign)
    assert np.array_equal(s, s_ref) and np.array_equal(q, q_ref)


def test_quantize_scalar_sequence_sweep():
    # the arithmetic contract itself: many thresholds, values straddling every rounding boundary
    rng = np.random.default_rng(77)
    for bits in (4, 8):
        qmax = 2 ** (bits - 1) - 1
        for T in rng.uniform(0.01, 50.0, 12).astype(np.float32):
            step = np.float32(T) / np.float32(qmax)
            k = rng.integers(-qmax - 2, qmax + 2, (64, 256))
            x = ((k + 0.5) * step).astype(np.float32)
            x = np.nextafter(x, rng.choice([-np.inf, np.inf], x.shape).astype(np.float32))
            x[::2] = ((k[::2] + 0.5) * step).astype(np.float32)
            q_ref, s_ref = ref.quantize(x, bits, threshold=float(T))
            q, s = gpu_quantize(x, bits, threshold=float(T))
            assert np.array_equal(s, s_ref)
            assert np.array_equal(q[:, :256], q_ref)


def test_quantize_denormals():
    x = np.array([[1e-40, -3e-39, 1e-38, 0.0, 5e-45, -1.4e-45, 2e-38, 1.1754944e-38]], dtype=np.float32)
    q_ref, s_ref = ref.quantize(x, 8, ldq=B.ocs_padded_cols(8))
    q, s = gpu_quantize(x, 8)
    assert np.array_equal(s, s_ref) and np.array_equal(q, q_ref)


# ---- ocs_select_channels ---------------------------------------------------------------------

@pytest.mark.parametrize("rows,C,g,s", [(5, 4, 1, 4), (9, 16, 4, 7), (64, 256, 1, 13), (33, 256, 9, 6),
                                        (17, 300, 3, 120), (40, 1024, 1, 103), (12, 2048, 1, 205),
                                        (8, 3000, 1, 150), (3, 1, 2, 5), (6, 7, 1, 0)])
@pytest.mark.parametrize("kind", ["heavy", "ties", "zero"])
def test_select_channels(rows, C, g, s, kind):
    rng = np.random.default_rng(rows + C + g + s)
    T = _tensor(rng, rows, C * g, kind)
    exp = ref.split_weights(T, C, g, s)
    got = gpu_select(T, C, g, s)
    assert np.array_equal(got["split_src"], exp["split_src"])
    assert np.array_equal(got["chan_src"], exp["chan_src"])
    assert np.array_equal(got["chan_depth"], exp["chan_depth"])
    assert got["max"] == exp["max"]


@pytest.mark.parametrize("E", [64, 65, 256, 257, 512, 513, 1024, 1025, 2048, 2049, 4096, 4097])
@pytest.mark.parametrize("kind", ["heavy", "ties"])
def test_select_at_the_list_layout_boundaries(E, kind):
    """C + s on either side of every size at which the selector changes how it deals the list
    over its lanes (slots per lane, one wave or four)."""
    s = 40
    rng = np.random.default_rng(E)
    T = _tensor(rng, 3, E - s, kind)
    exp = ref.split_weights(T, E - s, 1, s)
    got = gpu_select(T, E - s, 1, s)
    for k in ("split_src", "chan_src", "chan_depth"):
        assert np.array_equal(got[k], exp[k]), k
    assert got["max"] == exp["max"]


def test_select_resplits_one_dominant_channel():
    rng = np.random.default_rng(2)
    T = rng.standard_normal((10, 12)).astype(np.float32)
    T[4, 7] = 1000.0
    exp = ref.split_weights(T, 12, 1, 9)
    got = gpu_select(T, 12, 1, 9)
    assert exp["chan_depth"].max() >= 3
    for k in ("split_src", "chan_src", "chan_depth"):
        assert np.array_equal(got[k], exp[k])


# ---- ocs_split_weights -----------------------------------------------------------------------

@pytest.mark.parametrize("N,C,g,s", [(7, 12, 1, 5), (40, 64, 9, 4), (256, 256, 1, 13), (100, 37, 4, 6),
                                     (64, 3, 49, 1), (33, 130, 1, 0)])
@pytest.mark.parametrize("bits,clip", [(8, 1.0), (4, 0.8)])
def test_split_weights_halve(N, C, g, s, bits, clip):
    rng = np.random.default_rng(N + C + g + s)
    W = (_tensor(rng, N, C * g, "heavy") * 0.05).astype(np.float32)
    exp = ref.split_weights(W, C, g, s)
    got = gpu_split_weights(W, C, g, s, bits=bits, clip_ratio=clip)
    for k in ("split_src", "chan_src", "chan_depth"):
        assert np.array_equal(got[k], exp[k]), k
    assert np.array_equal(got["T_out"], exp["T_out"])
    assert got["max"] == exp["max"]
    q_ref, s_ref = ref.quantize(exp["T_out"], bits, clip_ratio=clip, ldq=B.ocs_padded_cols((C + s) * g))
    assert np.array_equal(got["scale"], s_ref)
    assert np.array_equal(got["Wq"], q_ref)


@pytest.mark.parametrize("sel_inline", [-1, 0, 64])   # default limit / selector launch / selection in the code pass
@pytest.mark.parametrize("N,C,g,s,kind", [
    (7, 12, 1, 5, "heavy"), (40, 64, 9, 4, "heavy"), (256, 256, 9, 6, "normal"), (100, 37, 4, 16, "heavy"),
    (100, 37, 4, 17, "heavy"), (64, 3, 49, 1, "normal"), (33, 130, 1, 0, "normal"), (20, 250, 1, 6, "ties"),
    (20, 251, 1, 6, "ties"), (9, 500, 2, 12, "heavy"), (9, 501, 1, 12, "heavy"), (5, 1010, 1, 14, "normal"),
    (5, 1010, 1, 15, "normal"), (12, 16, 3, 40, "heavy"), (300, 8, 1, 9, "zero")])
def test_split_weights_codes_only_routes(N, C, g, s, kind, sel_inline):
    """Codes only (no fp32 copy): with few splits the selection runs inside the code pass, one launch
    instead of two; both routes must write the same lists, maximum, grid and codes."""
    rng = np.random.default_rng(N + C + g + s)
    W = (_tensor(rng, N, C * g, kind) * 0.05).astype(np.float32)
    exp = ref.split_weights(W, C, g, s)
    B.ocs_tune("sel_inline", sel_inline)
    try:
        got = gpu_split_weights(W, C, g, s, bits=7, clip_ratio=0.9, want_f32=False)
    finally:
        B.ocs_tune("sel_inline", -1)
    for k in ("split_src", "chan_src", "chan_depth"):
        assert np.array_equal(got[k], exp[k]), k
    assert got["max"] == exp["max"]
    q_ref, s_ref = ref.quantize(exp["T_out"], 7, clip_ratio=0.9, ldq=B.ocs_padded_cols((C + s) * g))
    assert np.array_equal(got["scale"], s_ref)
    assert np.array_equal(got["Wq"], q_ref)


def test_split_weights_dup_mode():
    rng = np.random.default_rng(8)
    N, C, g, s = 30, 20, 4, 6
    W = _tensor(rng, N, C * g, "normal")
    split_src = np.array([3, 3, 20, 7, 0, 23], dtype=np.int32)   # includes copies of copies
    exp = ref.split_weights(W, C, g, s, mode=ref.MODE_DUP, split_src=split_src)
    got = gpu_split_weights(W, C, g, s, mode=B.MODE_DUP, split_src=split_src, bits=6)
    assert np.array_equal(got["chan_src"], exp["chan_src"])
    assert np.array_equal(got["chan_depth"], exp["chan_depth"])
    assert np.array_equal(got["T_out"], exp["T_out"])
    assert got["max"] == exp["max"]
    q_ref, s_ref = ref.quantize(exp["T_out"], 6, ldq=B.ocs_padded_cols((C + s) * g))
    assert np.array_equal(got["scale"], s_ref) and np.array_equal(got["Wq"], q_ref)


# ---- ocs_split_weights_qa (Sec. 3.3) -----------------------------------------------------------

@pytest.mark.parametrize("N,C,g,s", [(7, 12, 1, 5), (40, 64, 9, 4), (256, 256, 1, 13), (100, 37, 4, 6),
                                     (3, 5, 1, 0), (33, 3, 49, 1), (20, 8, 2, 40), (64, 500, 1, 25)])
@pytest.mark.parametrize("bits,clip", [(8, 1.0), (4, 0.8), (5, 1.0)])
def test_split_weights_qa(N, C, g, s, bits, clip):
    rng = np.random.default_rng(N * 7 + C + g + s + bits)
    W = _tensor(rng, N, C * g, "heavy")
    exp = ref.split_weights_qa(W, C, g, s, bits, clip_ratio=clip, ldq=B.ocs_padded_cols((C + s) * g))
    got = gpu_split_weights_qa(W, C, g, s, bits=bits, clip_ratio=clip)
    for k in ("split_src", "chan_src", "chan_depth", "chan_path", "scale", "T_out"):
        assert np.array_equal(got[k], exp[k]), k
    assert np.array_equal(got["Wq"], exp["q"])
    only_codes = gpu_split_weights_qa(W, C, g, s, bits=bits, clip_ratio=clip, want_f32=False)
    assert np.array_equal(only_codes["Wq"], exp["q"])
    only_f32 = gpu_split_weights_qa(W, C, g, s, bits=bits, clip_ratio=clip, want_codes=False)
    assert np.array_equal(only_f32["T_out"], exp["T_out"])


@pytest.mark.parametrize("N,C,g,s,why", [
    (3, 7000, 20, 5, "rows of 35,025 dwords: too long for the per-row bit mask, one pass"),
    (3, 200, 49, 190, "more dwords touch a split channel than the workgroup's list holds"),
    (5, 1000, 4, 1, "a single split: all but a handful of dwords on the vector path"),
    (3, 1500, 2, 1400, "more listed dwords than the per-element table in LDS holds: list without it"),
    (1000, 300, 4, 12, "enough workgroups for some of them to take the listed dwords beside the stream"),
])
def test_split_weights_qa_code_only_routes(N, C, g, s, why):
    """The code-only call picks its route by the shape: every route gives the oracle's codes."""
    rng = np.random.default_rng(C + g + s)
    W = _tensor(rng, N, C * g, "heavy")
    exp = ref.split_weights_qa(W, C, g, s, 6, ldq=B.ocs_padded_cols((C + s) * g))
    got = gpu_split_weights_qa(W, C, g, s, bits=6, want_f32=False)
    for k in ("split_src", "chan_src", "chan_depth", "chan_path", "scale"):
        assert np.array_equal(got[k], exp[k]), k
    assert np.array_equal(got["Wq"], exp["q"]), why


def test_split_weights_qa_ties_and_dominant_channel():
    # exact ties of floor(x + 1/2) on a step-1 grid, and one channel split over and over
    col0 = np.concatenate([[28.0], np.arange(-27 * 16, 27 * 16 + 1, 3) / 16.0]).astype(np.float32)
    W = np.stack([col0, np.full_like(col0, 2.5)], axis=1)
    W[2:5, 1] = [-2.5, 3.5, -0.5]
    exp = ref.split_weights_qa(W, 2, 1, 3, 4, ldq=B.ocs_padded_cols(5))
    got = gpu_split_weights_qa(W, 2, 1, 3, bits=4)
    assert np.array_equal(got["Wq"], exp["q"]) and np.array_equal(got["T_out"], exp["T_out"])
    assert np.array_equal(got["Wq"][:, [0, 2, 3, 4]].astype(np.int64).sum(axis=1),
                          np.floor(W[:, 0].astype(np.float64) + 0.5).astype(np.int64))
    dom = np.zeros((4, 6), dtype=np.float32)
    dom[1, 2] = 1.0
    exp = ref.split_weights_qa(dom, 6, 1, 40, 8, ldq=B.ocs_padded_cols(46))
    got = gpu_split_weights_qa(dom, 6, 1, 40, bits=8)
    for k in ("split_src", "chan_src", "chan_depth", "chan_path", "scale", "T_out"):
        assert np.array_equal(got[k], exp[k]), k
    assert np.array_equal(got["Wq"], exp["q"])


def test_qa_layer_end_to_end():
    # duplicated activations (Eq. 3) x QA-split weights through the GEMM, against the oracle chain
    rng = np.random.default_rng(5)
    M, C, g, N, s = 70, 48, 4, 33, 5
    X = _tensor(rng, M, C * g, "heavy")
    W = _tensor(rng, N, C * g, "heavy")
    ldq = B.ocs_padded_cols((C + s) * g)
    w_ref = ref.split_weights_qa(W, C, g, s, 5, ldq=ldq)
    xq_ref, sx_ref, _ = ref.split_act(X, C, g, w_ref["chan_src"], None, s, 8, ldq=ldq)
    acc_ref, y_ref = ref.qgemm(xq_ref, w_ref["q"], (C + s) * g, sx_ref[1], w_ref["scale"][1])
    w_gpu = gpu_split_weights_qa(W, C, g, s, bits=5)
    xq, sx = gpu_split_act(X, C, g, w_gpu["chan_src"], None, s, 8)
    acc, Y = gpu_qgemm(xq, w_gpu["Wq"], (C + s) * g, sx, w_gpu["scale"], bits_w=5)
    assert np.array_equal(acc, acc_ref)
    assert_y_close(Y, y_ref)


# ---- ocs_mse_clip_threshold (Sec. 4.1) ---------------------------------------------------------

@pytest.mark.parametrize("rows,cols,ld_extra", [(1, 1, 0), (64, 256, 0), (33, 147, 5), (257, 2304, 0), (700, 333, 3)])
@pytest.mark.parametrize("bits,n_bins,n_cand", [(4, 2048, 512), (8, 2048, 512), (6, 64, 7), (3, 1, 1), (5, 8192, 300)])
def test_mse_clip_threshold(rows, cols, ld_extra, bits, n_bins, n_cand):
    rng = np.random.default_rng(rows + cols + bits)
    x = _tensor(rng, rows, cols, "heavy")
    exp = ref.mse_clip(x, bits, n_bins=n_bins, n_cand=n_cand)
    got = gpu_mse_clip(x, bits, n_bins=n_bins, n_cand=n_cand, ld_extra=ld_extra)
    assert got["max"] == exp["max"]
    assert np.array_equal(got["hist"], exp["hist"])
    assert np.array_equal(got["mse"], exp["mse"])          # same operations in the same order
    assert got["threshold"] == exp["threshold"]


def test_mse_clip_threshold_degenerate_and_large():
    z = np.zeros((5, 9), dtype=np.float32)
    got = gpu_mse_clip(z, 8, n_bins=16, n_cand=4)
    assert got["threshold"] == 0.0 and got["max"] == 0.0 and got["hist"][0] == 45 and not got["mse"].any()
    ties = _tensor(np.random.default_rng(3), 61, 333, "ties")
    exp, got = ref.mse_clip(ties, 5, n_bins=128, n_cand=64), gpu_mse_clip(ties, 5, n_bins=128, n_cand=64)
    assert np.array_equal(got["hist"], exp["hist"]) and np.array_equal(got["mse"], exp["mse"])
    assert got["threshold"] == exp["threshold"]
    rng = np.random.default_rng(11)
    big = np.abs(rng.standard_normal((12544, 2304))).astype(np.float32)      # the bench workload's shape
    exp, got = ref.mse_clip(big, 4), gpu_mse_clip(big, 4)
    assert np.array_equal(got["hist"], exp["hist"]) and np.array_equal(got["mse"], exp["mse"])
    assert got["threshold"] == exp["threshold"] < exp["max"]
    # the threshold feeds the quantizer
    q_ref, s_ref = ref.quantize(big[:300], 4, threshold=float(exp["threshold"]), ldq=B.ocs_padded_cols(2304))
    q, sc = gpu_quantize(big[:300], 4, threshold=float(got["threshold"]))
    assert np.array_equal(q, q_ref) and np.array_equal(sc, s_ref)


# ---- ocs_split_act ---------------------------------------------------------------------------

@pytest.mark.parametrize("M,C,g,s", [(5, 8, 1, 3), (70, 64, 9, 4), (129, 256, 1, 13), (33, 37, 4, 6),
                                     (300, 3, 49, 1), (64, 500, 1, 25), (17, 20, 3, 0), (1000, 16, 1, 1),
                                     (77, 2048, 1, 205), (50, 64, 4, 300), (9, 512, 9, 26)])
@pytest.mark.parametrize("halve", [False, True])
@pytest.mark.parametrize("threshold", [None, 3.0])
@pytest.mark.parametrize("act_map", [0, 1, 2, 3, 4, 5, 6])   # lanes over the output / the input; +2: 64-bit indices;
def test_split_act(M, C, g, s, halve, threshold, act_map):  # +4: Eq. 4's depths from the per-column table in LDS;
    # 6: the tile-ordered pass wherever it serves the case (static grid, un-scaled copies, rows from 64 values)
    rng = np.random.default_rng(M + C + g + s)
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(X if halve else _tensor(rng, 9, C * g, "heavy"), C, g, s)
    cs, cd = sel["chan_src"], (sel["chan_depth"] if halve else None)
    ldq = B.ocs_padded_cols((C + s) * g)
    q_ref, s_ref, _ = ref.split_act(X, C, g, cs, cd, s, 8, threshold=threshold, clip_ratio=0.9, ldq=ldq)
    B.ocs_tune("act_tile", 1 if act_map == 6 else 0)
    B.ocs_tune("act_np", 0)
    if act_map < 6:
        B.ocs_tune("act_map", act_map & 1)
        B.ocs_tune("act_wide", (act_map >> 1) & 1)
        B.ocs_tune("act_dep", act_map >> 2)
    try:
        q, sc = gpu_split_act(X, C, g, cs, cd, s, 8, threshold=threshold, clip_ratio=0.9)
    finally:
        B.ocs_tune("act_map", -1)
        B.ocs_tune("act_wide", 0)
        B.ocs_tune("act_dep", -1)
        B.ocs_tune("act_tile", -1)
        B.ocs_tune("act_np", -1)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("M,C,g,s,ld_extra", [(64, 64, 1, 0, 0), (65, 64, 1, 4, 0), (300, 3, 49, 1, 0), (130, 67, 1, 5, 48),
                                              (257, 256, 1, 13, 112), (100, 128, 9, 7, 0), (63, 191, 1, 64, 16),
                                              (70, 13, 9, 2, 64), (200, 512, 4, 26, 0), (90, 64, 4, 200, 0)])
@pytest.mark.parametrize("tile", [0, 1])
def test_split_act_tile_order(M, C, g, s, ld_extra, tile):
    """The tile-ordered pass against the oracle (and so against the flat pass, run on the same cases):
    left-over columns, ragged last row tile, pitches beyond the recommended one (zero padding up to
    the pitch), a split list with repeats."""
    rng = np.random.default_rng(M * 7 + C + g + s)
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(_tensor(rng, 9, C * g, "heavy"), C, g, s)
    ldq = B.ocs_padded_cols((C + s) * g) + ld_extra
    q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=2.0, ldq=ldq)
    B.ocs_tune("act_tile", tile)
    B.ocs_tune("act_np", 0)
    try:
        q, sc = gpu_split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=2.0, ldq=ldq)
    finally:
        B.ocs_tune("act_tile", -1)
        B.ocs_tune("act_np", -1)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("M,C,g,s,ld_extra", [(64, 64, 1, 0, 0), (65, 64, 1, 4, 0), (300, 3, 49, 1, 0), (130, 67, 1, 5, 48),
                                              (257, 256, 1, 13, 112), (100, 128, 9, 7, 0), (63, 191, 1, 64, 16),
                                              (70, 13, 9, 2, 64), (200, 512, 4, 26, 0), (90, 64, 4, 100, 0),
                                              (5, 1, 4, 0, 0), (3, 5, 1, 1, 0), (1000, 16, 1, 1, 0), (37, 512, 9, 26, 0),
                                              (21, 2048, 4, 60, 0), (19, 1250, 1, 100, 32)])
@pytest.mark.parametrize("loads", [-1, 1, 2, 3, 4, 5, 6, 7, 8])
def test_split_act_one_shot(M, C, g, s, ld_extra, loads):
    """The one-shot pass (whole rows per workgroup, all loads at once, tail from the codes in LDS)
    against the oracle: by shape (-1) and with every number of loads per lane forced (a shape that a
    given count cannot hold falls to the other passes, and is compared all the same): left-over
    columns (K % 4), rows at odd alignment, a ragged last workgroup, fewer rows than a workgroup
    takes, pitches beyond the recommended one, copies of copies' sources, the longest rows served."""
    rng = np.random.default_rng(M * 11 + C + g + s)
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(_tensor(rng, 9, C * g, "heavy"), C, g, s)
    ldq = B.ocs_padded_cols((C + s) * g) + ld_extra
    q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=2.0, ldq=ldq)
    B.ocs_tune("act_np", loads)
    try:
        q, sc = gpu_split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=2.0, ldq=ldq)
    finally:
        B.ocs_tune("act_np", -1)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("M,C,g,s", [(5, 8, 1, 3), (70, 64, 9, 4), (300, 3, 49, 1), (1000, 16, 1, 1), (77, 2048, 1, 103),
                                     (9, 512, 9, 26), (2100, 512, 1, 26), (4100, 1030, 1, 5)])
@pytest.mark.parametrize("clip", [1.0, 0.7])
def test_split_act_per_batch_grid_one_shot(M, C, g, s, clip):
    """The per-batch grid as large tensors take it: max|X| as one value per workgroup, folded into one
    word by a launch of its own, then the split+quantize pass in its one-shot form with the clip ratio
    times that word as its threshold.  Twice in a row on the same scratch space, the second tensor
    with a smaller maximum (anything left over from the first call would show)."""
    rng = np.random.default_rng(M + 3 * C + g + s)
    sel = ref.split_weights(_tensor(rng, 9, C * g, "heavy"), C, g, s)
    ldq = B.ocs_padded_cols((C + s) * g)
    B.ocs_tune("max_flat", 2)
    try:
        for scale in (1.0, 0.25):
            X = _tensor(rng, M, C * g, "heavy") * np.float32(scale)
            q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=None, clip_ratio=clip, ldq=ldq)
            q, sc = gpu_split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=None, clip_ratio=clip)
            assert np.array_equal(sc, s_ref)
            assert np.array_equal(q, q_ref)
    finally:
        B.ocs_tune("max_flat", -1)


@pytest.mark.parametrize("seed", list(range(24)))
def test_split_act_static_grid_random_shapes(seed):
    """The static-grid pass as the library dispatches it (one-shot, tile-ordered or flat, by shape) on
    seeded random shapes against the oracle: row lengths of every residue modulo 4 and 64, group
    sizes 1..9, split counts from none to more than the channels, pitches at and beyond the
    recommended one, a threshold inside the data's range (so both clipping ends occur)."""
    rng = np.random.default_rng(1000 + seed)
    g = int(rng.choice([1, 1, 2, 3, 4, 7, 9]))
    C = int(rng.integers(1, 700 // g + 2))
    s = int(rng.choice([0, 1, max(1, C // 20), max(1, C // 8), C + 3]))
    M = int(rng.choice([1, 7, 63, 64, 65, 200, 517, 1500]))
    ld_extra = int(rng.choice([0, 0, 16, 64, 240]))
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(_tensor(rng, 5, C * g, "heavy"), C, g, s)
    ldq = B.ocs_padded_cols((C + s) * g) + ld_extra
    thr = float(np.quantile(np.abs(X), 0.98)) if X.size > 4 else 1.0
    q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=thr, ldq=ldq)
    q, sc = gpu_split_act(X, C, g, sel["chan_src"], None, s, 8, threshold=thr, ldq=ldq)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(q, q_ref)


@pytest.mark.parametrize("act_dep", [0, 1])
def test_split_act_deep_halvings(act_dep):
    """Eq. 4 with depth lists no greedy run would produce (the call takes any list): factors down to
    2^-126, the denormal 2^-127 .. 2^-149, and zero beyond, on values up to 2^125.  The per-column depth table (one byte per column, 255 standing for anything
    larger) and the look-up in global memory agree with the oracle."""
    rng = np.random.default_rng(31)
    M, C, g, s = 40, 12, 3, 4
    chan_src = np.array(list(range(C)) + [2, 5, 7, 11], dtype=np.int32)
    chan_depth = np.array([0, 1, 50, 100, 126, 127, 130, 140, 150, 200, 255, 300, 50, 127, 140, 300], dtype=np.int32)
    X = _tensor(rng, M, C * g, "normal")
    for j in range(C):    # channel j holds values near 2^depth (up to 2^125), so its products spread over the grid
        X[:, j * g:(j + 1) * g] *= np.float32(2.0 ** min(int(chan_depth[j]), 125))
    ldq = B.ocs_padded_cols((C + s) * g)
    q_ref, s_ref, _ = ref.split_act(X, C, g, chan_src, chan_depth, s, 8, threshold=3.0, ldq=ldq)
    for j in (3, 4, 5, 13):   # factors 2^-100, 2^-126 and the denormal 2^-127 all spread over the grid
        assert len(np.unique(q_ref[:, j * g:(j + 1) * g])) > 20
    B.ocs_tune("act_dep", act_dep)
    try:
        q, sc = gpu_split_act(X, C, g, chan_src, chan_depth, s, 8, threshold=3.0)
    finally:
        B.ocs_tune("act_dep", -1)
    assert np.array_equal(sc, s_ref)
    assert np.array_equal(q, q_ref)


def test_split_weights_halvings_that_leave_the_normal_range():
    """Weights of a few 1e-38: the halvings of Eq. 3 push them below the normal range, where every
    halving rounds; the expanded fp32 weights and the codes equal the oracle's (which halves split by
    split) on every route of the weight path: codes only (selection inside the code pass), fp32 and
    codes (selector launch, streaming pass, fp32 materialisation)."""
    rng = np.random.default_rng(5)
    N, Cn, g, s = 23, 10, 3, 9
    bits = rng.integers(1, 0x00040000, (N, Cn * g)).astype(np.uint32)
    bits[:, 6:9] = rng.integers(0x01000000, 0x01800000, (N, g))
    W = (bits | (rng.integers(0, 2, bits.shape).astype(np.uint32) << 31)).view(np.float32)
    exp = ref.split_weights(W, Cn, g, s)
    assert exp["chan_depth"].max() >= 3
    for want_f32 in (False, True):
        got = gpu_split_weights(W, Cn, g, s, bits=8, want_f32=want_f32)
        q_ref, sc_ref = ref.quantize(exp["T_out"], 8, ldq=got["Wq"].shape[1])
        assert np.array_equal(got["split_src"], exp["split_src"]) and np.array_equal(got["chan_depth"], exp["chan_depth"])
        if want_f32:
            assert np.array_equal(got["T_out"].view(np.uint32), exp["T_out"].view(np.uint32))
        assert np.array_equal(got["scale"], sc_ref)
        assert np.array_equal(got["Wq"], q_ref)
        assert len(np.unique(got["Wq"])) > 3


# ---- ocs_qgemm -------------------------------------------------------------------------------

GEMM_TILES = [6, 7, 9, 10, 11, 12, 14, 16, 17, 18, 19, 23, 24, 25]     # every tile variant of the library


@pytest.mark.parametrize("tile", [-1] + GEMM_TILES)
@pytest.mark.parametrize("pitch", ["tight", "lines"])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (64, 256, 269), (130, 70, 64), (257, 129, 200), (300, 200, 80),
                                   (70, 1100, 135), (700, 300, 1035), (300, 520, 2358), (128, 128, 4842)])
def test_qgemm(tile, pitch, M, N, K):
    """Rows at the recommended pitch (for a short K that is the row rounded up to 16 bytes only: the next
    row's codes follow at once, and what the row lacks up to its last K-step must count as zeros) and at
    whole 128-byte lines (every ring variant then walks the short shapes too)."""
    rng = np.random.default_rng(M + N + K)
    ld = B.ocs_padded_cols(K) if pitch == "tight" else -(-K // 128) * 128
    if pitch == "lines" and ld == B.ocs_padded_cols(K):
        pytest.skip("same pitch as the tight case")
    Xq = np.zeros((M, ld), dtype=np.int8)
    Wq = np.zeros((N, ld), dtype=np.int8)
    Xq[:, :K] = rng.integers(-127, 128, (M, K))
    Wq[:, :K] = rng.integers(-127, 128, (N, K))
    sx = np.array([3.0, 3.0 / 127], dtype=np.float32)
    sw = np.array([0.7, 0.7 / 127], dtype=np.float32)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, K, sx[1], sw[1])
    B.ocs_tune("gemm_tile", tile)
    try:
        acc, Y = gpu_qgemm(Xq, Wq, K, sx, sw)
        _, Y2 = gpu_qgemm(Xq, Wq, K, sx, sw, want_acc=False)
    finally:
        B.ocs_tune("gemm_tile", -1)
    assert np.array_equal(acc, acc_ref)
    assert_y_close(Y, y_ref)
    assert np.array_equal(Y, Y2)


@pytest.mark.parametrize("parts", [2, 3, 4, 7])
@pytest.mark.parametrize("M,N,K", [(1, 1, 500), (130, 70, 448), (257, 129, 1035), (700, 300, 1035), (300, 520, 2358),
                                   (1000, 512, 4842)])
def test_qgemm_split_k(parts, M, N, K):
    """The K extent of every tile shared between `parts` workgroups: accumulators bit for bit those of
    the oracle (and so of the un-split call), outputs identical to the un-split call's; twice in a row
    on the same counters, and with a workspace full of garbage."""
    rng = np.random.default_rng(M + N + K + parts)
    ld = B.ocs_padded_cols(K)
    Xq = np.zeros((M, ld), dtype=np.int8)
    Wq = np.zeros((N, ld), dtype=np.int8)
    Xq[:, :K] = rng.integers(-127, 128, (M, K))
    Wq[:, :K] = rng.integers(-127, 128, (N, K))
    sx = np.array([3.0, 3.0 / 127], dtype=np.float32)
    sw = np.array([0.7, 0.7 / 127], dtype=np.float32)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, K, sx[1], sw[1])
    _, Y_plain = gpu_qgemm(Xq, Wq, K, sx, sw, want_acc=False)
    need = B.ocs_qgemm_split_k_workspace_bytes(M, N, K, parts)
    assert need == -(-M // 256) * -(-N // 256) * parts * 256 * 256 * 4
    Xd, Wd, sxd, swd = dev(Xq), dev(Wq), dev(sx), dev(sw)
    ws = torch.randint(0, 255, (need,), dtype=torch.uint8, device="cuda")
    for rep in range(2):
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        Y = torch.full((M, N), -7.0, dtype=torch.float32, device="cuda")
        B.ocs_qgemm_split_k(Xd, ld, Wd, ld, M, N, K, 8, 8, sxd, swd, acc if rep == 0 else None,
                            N if rep == 0 else 0, Y, N, parts, ws)
        if rep == 0:
            assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(host(Y), Y_plain)
    assert_y_close(host(Y), y_ref)


# ---- ocs_split_act_qgemm: the two calls as one launch -----------------------------------------

@pytest.mark.parametrize("M,C,g,s,N", [(1, 64, 1, 0, 1), (130, 64, 1, 4, 64), (300, 64, 9, 4, 64), (257, 256, 1, 13, 128),
                                       (700, 128, 9, 7, 128), (129, 512, 1, 26, 256), (200, 256, 9, 13, 250),
                                       (64, 1024, 1, 52, 70), (90, 64, 4, 200, 33), (128, 64, 2, 64, 256),
                                       (500, 2048, 4, 103, 256), (300, 3, 49, 1, 64), (100, 37, 4, 6, 70),
                                       (77, 100, 1, 5, 128), (65, 67, 1, 0, 256), (130, 191, 1, 64, 200),
                                       (70, 13, 9, 2, 64)])
@pytest.mark.parametrize("bits_w,variant,stride", [(4, -1, -1), (8, 1, 0), (8, 2, 0), (4, -1, 37), (8, 2, 100)])
def test_split_act_qgemm(M, C, g, s, N, bits_w, variant, stride):   # variants: both workgroup shapes for N > 128;
    # stride: rows between workgroups by shape (-1: with so few rows, half-idle tiles), whole tiles (0), forced
    """X -> codes -> accumulators in one launch: the accumulators are bit for bit the oracle's GEMM on the
    oracle's codes of the expanded X, the outputs within the contract of the two-call path; weights at
    the recommended pitch (for a short K the rows end inside the last K-step)."""
    rng = np.random.default_rng(M + C + g + s + N)
    K = C * g
    X = np.abs(_tensor(rng, M, K, "heavy"))
    W = _tensor(rng, N, K, "normal") * np.float32(0.05)
    exp = ref.split_weights(W, C, g, s)
    # (a split list with repeats of one channel, as the greedy produces on heavy tails)
    Ke = (C + s) * g
    ldq = B.ocs_padded_cols(Ke)
    Wq, sw = ref.quantize(exp["T_out"], bits_w, clip_ratio=0.9, ldq=ldq)
    T = 3.0
    Xq, sx, _ = ref.split_act(X, C, g, exp["chan_src"], None, s, 8, threshold=T, ldq=ldq)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, Ke, sx[1], sw[1])
    assert B.ocs_split_act_qgemm_fits(M, C, g, s, N, K)
    Xd, Wd, swd = dev(X), dev(Wq), dev(sw)
    cs = dev(exp["chan_src"])
    th = torch.tensor([T], dtype=torch.float32, device="cuda")
    B.ocs_tune("fused_variant", variant)
    B.ocs_tune("fused_stride", stride)
    try:
        for want_acc in (True, False):
            acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda") if want_acc else None
            Y = torch.full((M, N), -7.0, dtype=torch.float32, device="cuda")
            sxo = torch.zeros(2, dtype=torch.float32, device="cuda")
            B.ocs_split_act_qgemm(Xd, M, C, g, K, cs, s, 8, th, Wd, ldq, N, bits_w, swd, sxo, acc,
                                  N if want_acc else 0, Y, N)
            if want_acc:
                assert np.array_equal(host(acc), acc_ref)
            assert np.array_equal(host(sxo), sx)
            assert_y_close(host(Y), y_ref)
    finally:
        B.ocs_tune("fused_variant", -1)
        B.ocs_tune("fused_stride", -1)


def test_split_act_qgemm_equals_the_two_calls_bit_for_bit():
    """Same Y bits as ocs_split_act followed by ocs_qgemm, on a shape that spans several row tiles with a
    ragged last one and has a channel split three times."""
    rng = np.random.default_rng(77)
    M, C, g, s, N = 1000, 128, 9, 9, 200
    K, Ke = C * g, (C + s) * g
    X = np.abs(_tensor(rng, M, K, "heavy"))
    W = _tensor(rng, N, K, "normal")
    W[:, 5 * g:6 * g] *= np.float32(40.0)          # one dominant channel: split again and again
    wts = gpu_split_weights(W, C, g, s, bits=4, want_f32=False)
    assert wts["chan_depth"].max() >= 3
    ldq = wts["Wq"].shape[1]
    Xq, sx = gpu_split_act(X, C, g, wts["chan_src"], None, s, 8, threshold=2.5, ldq=ldq)
    _, Y2 = gpu_qgemm(Xq, wts["Wq"], Ke, sx, wts["scale"], want_acc=False)
    Y = torch.full((M, N), -7.0, dtype=torch.float32, device="cuda")
    B.ocs_split_act_qgemm(dev(X), M, C, g, K, dev(wts["chan_src"]), s, 8,
                          torch.tensor([2.5], dtype=torch.float32, device="cuda"), dev(wts["Wq"]), ldq, N, 4,
                          dev(wts["scale"]), None, None, 0, Y, N)
    assert np.array_equal(host(Y), Y2)


def test_qgemm_extreme_codes_do_not_overflow():
    K = 4096
    Xq = np.full((40, K), 127, dtype=np.int8)
    Wq = np.full((50, K), -127, dtype=np.int8)
    Wq[::2] = 127
    sx = np.array([1.0, 1.0 / 127], dtype=np.float32)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, K, sx[1], sx[1])
    acc, Y = gpu_qgemm(Xq, Wq, K, sx, sx)
    assert np.array_equal(acc, acc_ref)
    assert_y_close(Y, y_ref)


# ---- ocs_qconv: the lowering of a convolution inside the GEMM's operand loader ---------------------

def _conv_reference(A, Wm, Cn, kh, kw, stride, pad, s, bits_x, bits_w, threshold):
    Bn, H, W, _ = A.shape
    g, E = kh * kw, Cn + s
    sp = ref.split_weights(Wm, Cn, g, s)
    ldq = B.ocs_padded_cols(E * g)
    Wq, sw = ref.quantize(sp["T_out"], bits_w, ldq=ldq)
    Aq, sx, _ = ref.split_act(A.reshape(-1, Cn), Cn, 1, sp["chan_src"], None, s, bits_x, threshold=threshold)
    Xq = np.zeros((ref.conv_out_size(H, kh, stride, pad) * ref.conv_out_size(W, kw, stride, pad) * Bn, ldq),
                  dtype=np.int8)
    Xq[:, :E * g] = ref.im2col(Aq.reshape(Bn, H, W, E), kh, kw, stride, pad)
    acc, Y = ref.qgemm(Xq, Wq, E * g, sx[1], sw[1])
    return dict(acc=acc, Y=Y, Aq=Aq, sx=sx, Wq=Wq, sw=sw)


@pytest.mark.parametrize("tile", [-1, 6, 7, 9, 10, 12])
@pytest.mark.parametrize("Bn,H,W,Cn,N,kh,kw,stride,pad,s", [
    (2, 14, 14, 64, 96, 3, 3, 1, 1, 4),        # the common 3x3
    (3, 9, 7, 20, 33, 3, 3, 2, 1, 2),          # stride 2, ragged everything
    (2, 8, 8, 128, 70, 1, 1, 1, 0, 7),         # 1x1
    (2, 9, 9, 64, 64, 1, 1, 2, 0, 4),          # 1x1 stride 2: skips pixels
    (1, 23, 17, 3, 64, 7, 7, 2, 3, 1),         # stem-like: 3 channels, 7x7
    (1, 5, 6, 130, 40, 2, 3, 1, 0, 0),         # no split, no padding; 9 chunks per pixel: K-steps straddle taps
    (2, 6, 6, 10, 50, 3, 3, 1, 1, 1),          # one chunk per pixel: four taps per K-step
    (4, 14, 14, 256, 256, 3, 3, 1, 1, 6),      # config 2's layer at batch 4
])
def test_qconv(tile, Bn, H, W, Cn, N, kh, kw, stride, pad, s):
    rng = np.random.default_rng(Bn + H + W + Cn + N + kh + stride + s)
    A = _tensor(rng, Bn * H * W, Cn, "heavy").reshape(Bn, H, W, Cn)
    Wm = _tensor(rng, N, Cn * kh * kw, "heavy")
    exp = _conv_reference(A, Wm, Cn, kh, kw, stride, pad, s, 8, 6, None)
    B.ocs_tune("gemm_tile", tile)
    try:
        got = gpu_conv_layer(A, Wm, Cn, kh, kw, stride, pad, s, bits_x=8, bits_w=6)
    finally:
        B.ocs_tune("gemm_tile", -1)
    E, ldc = Cn + s, got["ldc"]
    assert np.array_equal(got["sx"], exp["sx"]) and np.array_equal(got["sw"], exp["sw"])
    assert np.array_equal(got["Aq"][:, :E], exp["Aq"][:, :E]) and not got["Aq"][:, E:].any()
    # tap-major weights: Wt[n, t*ldc + j] = Wq[n, j*g + t], zero padding, zero last row
    g = kh * kw
    assert ldc == (E + 15) // 16 * 16 and got["Wt"].shape[1] == (g * ldc + 63) // 64 * 64
    Wt = got["Wt"][:, :g * ldc].reshape(N + 1, g, ldc)
    assert np.array_equal(Wt[:N, :, :E], exp["Wq"][:, :E * g].reshape(N, E, g).transpose(0, 2, 1))
    assert not Wt[:N, :, E:].any() and not Wt[N].any() and not got["Wt"][:, g * ldc:].any()
    assert np.array_equal(got["acc"], exp["acc"])
    assert_y_close(got["Y"], exp["Y"])


def test_qconv_equals_the_lowered_gemm_path():
    # same layer through ocs_split_act on the im2col matrix + ocs_qgemm, with a static grid
    rng = np.random.default_rng(99)
    Bn, H, W, Cn, N, s = 2, 10, 10, 48, 80, 3
    A = np.abs(_tensor(rng, Bn * H * W, Cn, "normal")).reshape(Bn, H, W, Cn)
    Wm = _tensor(rng, N, Cn * 9, "heavy")
    got = gpu_conv_layer(A, Wm, Cn, 3, 3, 1, 1, s, threshold=4.0)
    X = ref.im2col(A, 3, 3, 1, 1)
    xq, sx = gpu_split_act(X, Cn, 9, got["chan_src"], None, s, 8, threshold=4.0)
    acc, Y = gpu_qgemm(xq, got["Wq"], (Cn + s) * 9, sx, got["sw"])
    assert np.array_equal(got["acc"], acc) and np.array_equal(got["Y"], Y)


@pytest.mark.parametrize("tile", [-1, 11, 23, 24, 25])
@pytest.mark.parametrize("ldx_extra,ldw_extra", [(0, 0), (64, 0), (0, 64), (64, 64), (192, 128)])
@pytest.mark.parametrize("M,N,K", [(130, 140, 180), (300, 260, 2358)])
def test_qgemm_k_step_of_128_needs_both_paddings(tile, ldx_extra, ldw_extra, M, N, K):
    """K rounded up to 64 is an odd multiple of 64 here.  The tiles with a 128-byte K-step may
    take the next 64 bytes in only when both leading dimensions hold them (zero padding); the
    rows of a tensor whose leading dimension stops at the 64-byte boundary are followed directly
    by the next row's codes, which must not enter the sum."""
    rng = np.random.default_rng(M + N + K + ldx_extra)
    k64 = (K + 63) // 64 * 64
    assert k64 % 128 == 64
    Xq = np.zeros((M, k64 + ldx_extra), dtype=np.int8)
    Wq = np.zeros((N, k64 + ldw_extra), dtype=np.int8)
    Xq[:, :K] = rng.integers(-127, 128, (M, K))
    Wq[:, :K] = rng.integers(-127, 128, (N, K))
    sx = np.array([3.0, 3.0 / 127], dtype=np.float32)
    sw = np.array([0.7, 0.7 / 127], dtype=np.float32)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, K, sx[1], sw[1])
    B.ocs_tune("gemm_tile", tile)
    try:
        acc, Y = gpu_qgemm(Xq, Wq, K, sx, sw)
    finally:
        B.ocs_tune("gemm_tile", -1)
    assert np.array_equal(acc, acc_ref)
    assert_y_close(Y, y_ref)


# ---- output handed to the next layer as codes ----------------------------------------------------

def _next_layer_list(rng, N, s_next):
    nxt = ref.split_weights(rng.standard_normal((5, N)).astype(np.float32), N, 1, s_next)
    return nxt["chan_src"]


@pytest.mark.parametrize("tile", [-1] + GEMM_TILES)
@pytest.mark.parametrize("M,N,K,s_next,relu", [(1, 1, 1, 0, False), (130, 70, 64, 9, True), (257, 129, 200, 0, False),
                                               (300, 520, 2358, 26, True), (700, 300, 269, 15, False)])
def test_qgemm_requant(tile, M, N, K, s_next, relu):
    rng = np.random.default_rng(M + N + K + s_next)
    ld = B.ocs_padded_cols(K)
    Xq = np.zeros((M, ld), dtype=np.int8)
    Wq = np.zeros((N, ld), dtype=np.int8)
    Xq[:, :K] = rng.integers(-127, 128, (M, K))
    Wq[:, :K] = rng.integers(-31, 32, (N, K))
    sx = np.array([3.0, 3.0 / 127], dtype=np.float32)
    sw = np.array([0.7, 0.7 / 31], dtype=np.float32)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, K, sx[1], sw[1])
    T = float(np.float32(0.5 * np.abs(y_ref).max())) if np.abs(y_ref).max() > 0 else 1.0
    cs = _next_layer_list(rng, N, s_next) if s_next else None
    ldy = B.ocs_padded_channels(N + s_next) + 16
    q_ref, sc_ref = ref.requantize(acc_ref, sx[1], sw[1], T, 5, cs, s_next, relu=relu, ldq=ldy)
    Yq = torch.full((M, ldy), 77, dtype=torch.int8, device="cuda")     # the call writes its pad columns itself
    acc = torch.full((M, N), -9, dtype=torch.int32, device="cuda")
    sc = torch.zeros(2, dtype=torch.float32, device="cuda")
    thr = torch.tensor([T], dtype=torch.float32, device="cuda")
    B.ocs_tune("gemm_tile", tile)
    try:
        B.ocs_qgemm_requant(dev(Xq), ld, dev(Wq), ld, M, N, K, 8, 6, dev(sx), dev(sw), relu, thr, 5,
                            None if cs is None else dev(cs), s_next, Yq, ldy, sc, acc, N)
    finally:
        B.ocs_tune("gemm_tile", -1)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(sc), sc_ref)
    assert np.array_equal(host(Yq), q_ref)


@pytest.mark.parametrize("tile", [-1, 6, 10])
def test_conv_chain_with_codes_between_the_layers(tile):
    # 3x3 convolution -> ReLU -> codes -> 1x1 layer (a GEMM on those codes), against the oracle
    rng = np.random.default_rng(17 + tile)
    Bn, H, W, C1, N1, N2, s1, s2 = 2, 9, 8, 24, 40, 36, 3, 4
    A = _tensor(rng, Bn * H * W, C1, "heavy").reshape(Bn, H, W, C1)
    W1 = _tensor(rng, N1, C1 * 9, "heavy")
    W2 = _tensor(rng, N2, N1, "heavy")
    # oracle: layer 1
    first = _conv_reference(A, W1, C1, 3, 3, 1, 1, s1, 8, 6, None)
    sp2 = ref.split_weights(W2, N1, 1, s2)
    ld2 = B.ocs_padded_cols(N1 + s2)
    W2q, sw2 = ref.quantize(sp2["T_out"], 6, ldq=ld2)
    T2 = float(np.float32(0.4) * np.float32(np.abs(first["Y"]).max()))
    X2q, sx2 = ref.requantize(first["acc"], first["sx"][1], first["sw"][1], T2, 8, sp2["chan_src"], s2, relu=True, ldq=ld2)
    acc2_ref, y2_ref = ref.qgemm(X2q, W2q, N1 + s2, sx2[1], sw2[1])
    # GPU: layer 1 with the re-quantizing epilogue, layer 2 a plain GEMM on its codes
    g1 = gpu_conv_layer(A, W1, C1, 3, 3, 1, 1, s1, bits_x=8, bits_w=6)
    w2 = gpu_split_weights(W2, N1, 1, s2, bits=6, want_f32=False)
    assert np.array_equal(w2["Wq"], W2q) and np.array_equal(w2["chan_src"], sp2["chan_src"])
    M = Bn * H * W
    Yq = torch.full((M, ld2), 77, dtype=torch.int8, device="cuda")
    sc2 = torch.zeros(2, dtype=torch.float32, device="cuda")
    thr = torch.tensor([T2], dtype=torch.float32, device="cuda")
    Wt = dev(g1["Wt"])
    B.ocs_tune("gemm_tile", tile)
    try:
        B.ocs_qconv_requant(dev(g1["Aq"]), g1["ldc"], Bn, H, W, C1 + s1, 3, 3, 1, 1, Wt, N1, 8, 6, dev(g1["sx"]),
                            dev(g1["sw"]), True, thr, 8, dev(sp2["chan_src"]), s2, Yq, ld2, sc2)
    finally:
        B.ocs_tune("gemm_tile", -1)
    assert np.array_equal(host(sc2), sx2) and np.array_equal(host(Yq), X2q)
    acc2, Y2 = gpu_qgemm(host(Yq), w2["Wq"], N1 + s2, host(sc2), w2["scale"], bits_w=6)
    assert np.array_equal(acc2, acc2_ref)
    assert_y_close(Y2, y2_ref)


# ---- seeded random layers through the whole chain -------------------------------------------------

@pytest.mark.parametrize("seed", range(24))
def test_random_layer_end_to_end(seed):
    from paper_1901_09504_amd.layer import ExpandedLayer
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.integers(1, 400))
    C = int(rng.integers(1, 300))
    g = int(rng.choice([1, 1, 2, 4, 9]))
    N = int(rng.integers(1, 300))
    r = float(rng.choice([0.0, 0.01, 0.05, 0.1, 0.3]))
    bits_w, bits_x = int(rng.integers(2, 9)), int(rng.integers(2, 9))
    clip = float(rng.choice([1.0, 0.9, 0.5]))
    kind = str(rng.choice(["heavy", "normal", "ties"]))
    X, W = _tensor(rng, M, C * g, kind), _tensor(rng, N, C * g, "heavy")
    static = None if seed % 3 else float(np.float32(0.7 * np.abs(X).max() + 1e-3))
    L = ExpandedLayer(N, C, g, r, bits_w, bits_x, clip_ratio_w=clip)
    L.prepare_weights(dev(W))
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    th = None if static is None else torch.tensor([static], dtype=torch.float32, device="cuda")
    Y = L.forward(dev(X), threshold=th, acc_out=acc)
    sp = ref.split_weights(W, C, g, L.s)
    Wq, sw = ref.quantize(sp["T_out"], bits_w, clip_ratio=clip, ldq=L.ldq)
    Xq, sx, _ = ref.split_act(X, C, g, sp["chan_src"], None, L.s, bits_x, threshold=static, ldq=L.ldq)
    acc_ref, y_ref = ref.qgemm(Xq, Wq, L.Ke, sx[1], sw[1])
    assert np.array_equal(host(L.split_src)[:L.s], sp["split_src"])
    assert np.array_equal(host(L.Wq), Wq) and np.array_equal(host(L.Xq[:M]), Xq)
    assert np.array_equal(host(L.scale_w), sw) and np.array_equal(host(L.scale_x), sx)
    assert np.array_equal(host(acc), acc_ref)
    assert_y_close(host(Y), y_ref)
    # the same layer un-expanded on folded codes, when they fit
    worst = int(host(L.fold_weights())[0])
    Wf_ref, worst_ref = ref.fold_weights(Wq, C, g, L.s, sp["chan_src"], ldf=L.ldf)
    assert worst == worst_ref and np.array_equal(host(L.Wf), Wf_ref)
    if worst <= 127:
        acc_f = torch.empty((M, N), dtype=torch.int32, device="cuda")
        Y_e = Y.clone()
        Y_f = L.forward_folded(dev(X), threshold=th, acc_out=acc_f)
        assert torch.equal(acc, acc_f) and torch.equal(Y_e, Y_f)


@pytest.mark.parametrize("seed", range(12))
def test_random_convolution(seed):
    rng = np.random.default_rng(2000 + seed)
    kh, kw = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
    H, W = int(rng.integers(max(1, kh - 2 * pad), 13)), int(rng.integers(max(1, kw - 2 * pad), 13))
    Bn, Cn, N = int(rng.integers(1, 4)), int(rng.integers(1, 90)), int(rng.integers(1, 150))
    s = int(rng.integers(0, 6))
    A = _tensor(rng, Bn * H * W, Cn, "heavy").reshape(Bn, H, W, Cn)
    Wm = _tensor(rng, N, Cn * kh * kw, "heavy")
    exp = _conv_reference(A, Wm, Cn, kh, kw, stride, pad, s, 8, 5, None)
    got = gpu_conv_layer(A, Wm, Cn, kh, kw, stride, pad, s, bits_x=8, bits_w=5)
    assert np.array_equal(got["acc"], exp["acc"])
    assert_y_close(got["Y"], exp["Y"])


# ---- paths that ordinary shapes do not reach --------------------------------------------------------

def test_expanded_channel_limit_and_long_tails():
    # C + s at the library's limit of 8000 expanded channels (the selector's list fills its LDS)
    rng = np.random.default_rng(7)
    T = _tensor(rng, 3, 7000, "heavy")
    exp = ref.split_weights(T, 7000, 1, 1000)
    got = gpu_select(T, 7000, 1, 1000)
    for k in ("split_src", "chan_src", "chan_depth"):
        assert np.array_equal(got[k], exp[k]), k
    # more appended + padded columns than the split+quantize kernels keep in their LDS table
    M, C, g, s = 12, 30, 9, 260
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(_tensor(rng, 5, C * g, "heavy"), C, g, s)
    ldq = B.ocs_padded_cols((C + s) * g)
    for cd in (None, sel["chan_depth"]):
        q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], cd, s, 7, ldq=ldq)
        for wide in (0, 1):
            B.ocs_tune("act_wide", wide)
            try:
                q, sc = gpu_split_act(X, C, g, sel["chan_src"], cd, s, 7)
            finally:
                B.ocs_tune("act_wide", 0)
            assert np.array_equal(sc, s_ref) and np.array_equal(q, q_ref)


def test_streaming_hint_and_many_weight_rows():
    rng = np.random.default_rng(8)
    # non-temporal loads of X in the split+quantize pass (a launch option)
    M, C, g, s = 200, 64, 9, 4
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(_tensor(rng, 9, C * g, "heavy"), C, g, s)
    q_ref, s_ref, _ = ref.split_act(X, C, g, sel["chan_src"], None, s, 8, ldq=B.ocs_padded_cols((C + s) * g))
    B.ocs_tune("act_nt", 1)
    try:
        q, sc = gpu_split_act(X, C, g, sel["chan_src"], None, s, 8)
    finally:
        B.ocs_tune("act_nt", 0)
    assert np.array_equal(sc, s_ref) and np.array_equal(q, q_ref)
    # more weight rows than one launch of the fp32 expansion covers (65535 per launch)
    N, C, g, s = 70000, 4, 1, 2
    W = _tensor(rng, N, C * g, "normal")
    exp = ref.split_weights(W, C, g, s)
    got = gpu_split_weights(W, C, g, s, bits=6)
    assert np.array_equal(got["T_out"], exp["T_out"])
    q_ref, sw_ref = ref.quantize(exp["T_out"], 6, ldq=B.ocs_padded_cols((C + s) * g))
    assert np.array_equal(got["Wq"], q_ref) and np.array_equal(got["scale"], sw_ref)


# ---- ocs_split_act_qa: Sec. 3.3 on the activation side -----------------------------------------------

@pytest.mark.parametrize("M,C,g,s", [(5, 8, 1, 3), (70, 64, 9, 4), (129, 256, 1, 13), (33, 37, 4, 6), (17, 20, 3, 0),
                                     (64, 500, 1, 25), (9, 12, 1, 30)])
@pytest.mark.parametrize("bits", [4, 8])
def test_split_act_qa(M, C, g, s, bits):
    rng = np.random.default_rng(M + C + g + s + bits)
    X = _tensor(rng, M, C * g, "heavy")
    sel = ref.split_weights(X, C, g, s)                       # the choice made on the batch
    T = float(np.float32(sel["max"]))
    ldq = B.ocs_padded_cols((C + s) * g)
    q_ref, s_ref, _ = ref.split_act_qa(X, C, g, sel["split_src"], s, bits, T, ldq=ldq)
    Xd = dev(X)
    cp = torch.full((C + s,), -7, dtype=torch.int32, device="cuda")
    q = torch.full((M, ldq), 77, dtype=torch.int8, device="cuda")
    sc = torch.zeros(2, dtype=torch.float32, device="cuda")
    ss = dev(sel["split_src"]) if s > 0 else None
    B.ocs_split_act_qa(Xd, M, C, g, Xd.stride(0), ss, dev(sel["chan_src"]), dev(sel["chan_depth"]), cp, s, bits,
                       torch.tensor([T], dtype=torch.float32, device="cuda"), q, ldq, sc)
    assert np.array_equal(host(sc), s_ref)
    assert np.array_equal(host(q), q_ref)
    wq = ref.split_weights_qa(X, C, g, s, bits)               # same list, same histories
    assert np.array_equal(host(cp).view(np.uint32), wq["chan_path"])


def test_activation_ocs_with_qa_members_end_to_end():
    from paper_1901_09504_amd import workloads as wl
    from paper_1901_09504_amd.layer import ExpandedLayer
    (layer,) = wl.config(1)
    W, X = wl.weights(layer), wl.activations(layer)
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x)
    acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
    Y = L.forward_act_ocs(dev(W), dev(X), acc_out=acc, qa=True)
    sel = ref.split_weights(X, layer.C, layer.g, L.s)
    dup = ref.split_weights(W, layer.C, layer.g, L.s, mode=ref.MODE_DUP, split_src=sel["split_src"])
    Xq_ref, sx_ref, _ = ref.split_act_qa(X, layer.C, layer.g, sel["split_src"], L.s, layer.bits_x,
                                         float(np.float32(sel["max"])), ldq=L.ldq)
    Wq_ref, sw_ref = ref.quantize(dup["T_out"], layer.bits_w, ldq=L.ldq)
    assert np.array_equal(host(L.Xq[:layer.M]), Xq_ref) and np.array_equal(host(L.scale_x), sx_ref)
    assert np.array_equal(host(L.Wq), Wq_ref)
    acc_ref, y_ref = ref.qgemm(Xq_ref, Wq_ref, L.Ke, sx_ref[1], sw_ref[1])
    assert np.array_equal(host(acc), acc_ref)
    assert_y_close(host(Y), y_ref)
