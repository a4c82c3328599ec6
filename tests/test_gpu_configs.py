"""GPU parity on the five synthetic configurations, end to end through the C ABI:
off-line weight path (select, halve, clip, quantize), per-batch activation path
(duplicate / halve, quantize) and the expanded integer GEMM with its dequantizing epilogue.

Every expected value comes from the CPU oracle on the same seeded inputs.  Where the layer
is too large for the oracle's GEMM to finish in seconds, the GPU still runs the full layer in
its normal launch configuration and the oracle recomputes a sample of complete rows (rows of
the output are independent once the scales are fixed): the first and last row blocks, which
hold the ragged edge, plus seeded random rows."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1901_09504_amd import binding as B
from paper_1901_09504_amd import workloads as wl
from paper_1901_09504_amd.layer import ExpandedLayer

from gpu_util import assert_y_close, dev, host, require_gpu

pytestmark = pytest.mark.gpu

FULL_ROWS = 26000      # up to this many rows the oracle recomputes every row (configs 1-4: all of them)
SAMPLED = 4096         # seeded random complete rows per larger layer, beside its first and last 256


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    require_gpu()


def _sample_rows(layer, n=SAMPLED):
    M = layer.M
    if M <= FULL_ROWS:
        return np.arange(M)
    rng = np.random.default_rng(layer.seed)
    head = np.arange(0, 256)
    tail = np.arange(M - 256, M)
    mid = rng.choice(np.arange(256, M - 256), size=n, replace=False)
    return np.unique(np.concatenate([head, mid, tail]))


def _activations(layer):
    if layer.M * layer.K < (1 << 24):
        return wl.activations(layer)
    # large tensors: the independent row blocks drawn on several threads (same values)
    return wl.activations_into(layer, np.empty((layer.M, layer.K), dtype=np.float32), threads=16)


def check_weight_path(layer, W, clip):
    """W1-W3 on the GPU against the literal one-split-at-a-time oracle.  Returns both sides."""
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, clip_ratio_w=clip)
    assert L.s == ref.num_splits(layer.C, layer.r)
    Wd = dev(W)
    L.prepare_weights(Wd)
    exp = ref.split_weights(W, layer.C, layer.g, L.s)
    q_ref, sw_ref = ref.quantize(exp["T_out"], layer.bits_w, clip_ratio=clip, ldq=L.ldq)
    assert np.array_equal(host(L.split_src)[:L.s], exp["split_src"])
    assert np.array_equal(host(L.chan_src), exp["chan_src"])
    assert np.array_equal(host(L.chan_depth), exp["chan_depth"])
    assert host(L.wmax)[0] == exp["max"]
    assert np.array_equal(host(L.scale_w), sw_ref)
    assert np.array_equal(host(L.Wq), q_ref)
    return L, exp, q_ref, sw_ref


def check_forward(layer, L, exp, Wq_ref, sw_ref, X_dev, X_rows, rows, threshold):
    """X2 + G1 + G2 on the GPU for the whole layer; the oracle recomputes `rows`."""
    M = layer.M
    th = None if threshold is None else torch.tensor([threshold], dtype=torch.float32, device="cuda")
    acc = torch.empty((M, layer.N), dtype=torch.int32, device="cuda")
    Y = L.forward(X_dev, threshold=th, acc_out=acc)
    Xq_ref, sx_ref, _ = ref.split_act(X_rows, layer.C, layer.g, exp["chan_src"], None, L.s, layer.bits_x,
                                      threshold=threshold, ldq=L.ldq)
    rows_t = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(L.scale_x), sx_ref)
    assert np.array_equal(host(L.Xq[:M][rows_t]), Xq_ref)
    acc_ref, y_ref = ref.qgemm(Xq_ref, Wq_ref, L.Ke, sx_ref[1], sw_ref[1])
    assert np.array_equal(host(acc[rows_t]), acc_ref)
    assert_y_close(host(Y[rows_t]), y_ref)
    # the timed configuration stores no accumulators: same outputs
    Y1 = Y.clone()
    Y2 = L.forward(X_dev, threshold=th)
    assert torch.equal(Y1, Y2)
    # split + quantize + GEMM as one launch, where that entry point serves the shape: the sampled
    # accumulators against the oracle again, and every output bit against the two launches
    if th is not None and L.fused_fits(X_dev):
        acc.fill_(-7)
        L.scale_x.zero_()
        Y3 = L.forward_fused(X_dev, th, acc_out=acc)
        assert np.array_equal(host(L.scale_x), sx_ref)
        assert np.array_equal(host(acc[rows_t]), acc_ref)
        assert torch.equal(Y1, Y3)
        Y3.fill_(-7.0)
        assert torch.equal(Y1, L.forward_fused(X_dev, th))      # no accumulators stored
    return sx_ref


def run_layer(layer, clips=(1.0,), dynamic=True, static_threshold=None):
    W = wl.weights(layer)
    rows = _sample_rows(layer)
    X = _activations(layer)
    X_dev = dev(X)
    first = True
    for clip in clips:
        L, exp, Wq_ref, sw_ref = check_weight_path(layer, W, clip)
        if not first:
            continue            # the activation path does not depend on the weight clip
        first = False
        if dynamic:
            # the dynamic grid spans the whole batch: the oracle's threshold is its own max over
            # all of X; the sampled rows are then requantized with that threshold
            T = float(np.float32(np.abs(X).max()))
            Xq_full, sx_full, _ = ref.split_act(X, layer.C, layer.g, exp["chan_src"], None, L.s,
                                                layer.bits_x, ldq=L.ldq)
            assert sx_full[0] == np.float32(T)
            acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
            Y = L.forward(X_dev, threshold=None, acc_out=acc)
            assert np.array_equal(host(L.scale_x), sx_full)
            assert np.array_equal(host(L.Xq[:layer.M]), Xq_full)
            acc_ref, y_ref = ref.qgemm(Xq_full[rows], Wq_ref, L.Ke, sx_full[1], sw_ref[1])
            rows_t = torch.from_numpy(rows).cuda()
            assert np.array_equal(host(acc[rows_t]), acc_ref)
            assert_y_close(host(Y[rows_t]), y_ref)
        if static_threshold is not None:
            check_forward(layer, L, exp, Wq_ref, sw_ref, X_dev, X[rows], rows, static_threshold)
    del X_dev
    torch.cuda.empty_cache()


# ---- config 1: single FC layer, weight OCS and activation OCS -------------------------------------

def test_config1_weight_ocs():
    (layer,) = wl.config(1)
    run_layer(layer, dynamic=True, static_threshold=6.0)


def test_config1_activation_ocs():
    (layer,) = wl.config(1)
    W, X = wl.weights(layer), wl.activations(layer)
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x)
    acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
    Y = L.forward_act_ocs(dev(W), dev(X), acc_out=acc)
    sel = ref.split_weights(X, layer.C, layer.g, L.s)                      # choice made on the batch
    dup = ref.split_weights(W, layer.C, layer.g, L.s, mode=ref.MODE_DUP, split_src=sel["split_src"])
    Xq_ref, sx_ref, _ = ref.split_act(X, layer.C, layer.g, sel["chan_src"], sel["chan_depth"], L.s,
                                      layer.bits_x, ldq=L.ldq)
    Wq_ref, sw_ref = ref.quantize(dup["T_out"], layer.bits_w, ldq=L.ldq)
    assert sel["chan_depth"].max() >= 1 and sx_ref[0] < np.abs(X).max()     # outliers were split
    assert np.array_equal(host(L.split_src)[:L.s], sel["split_src"])
    assert np.array_equal(host(L.chan_src), sel["chan_src"])
    assert np.array_equal(host(L.chan_depth), sel["chan_depth"])
    assert np.array_equal(host(L.scale_x), sx_ref) and np.array_equal(host(L.scale_w), sw_ref)
    assert np.array_equal(host(L.Xq[:layer.M]), Xq_ref)
    assert np.array_equal(host(L.Wq), Wq_ref)
    acc_ref, y_ref = ref.qgemm(Xq_ref, Wq_ref, L.Ke, sx_ref[1], sw_ref[1])
    assert np.array_equal(host(acc), acc_ref)
    assert_y_close(host(Y), y_ref)


# ---- config 2: the 3x3 convolution as an im2col GEMM, full size, every row ----------------------

def test_config2_full_size():
    (layer,) = wl.config(2)
    run_layer(layer, dynamic=True, static_threshold=5.5)


# ---- config 3: 1x1 convolutions, three expand ratios, 6-bit weights -------------------------------

@pytest.mark.parametrize("idx", range(9))
def test_config3(idx):
    layer = wl.config(3)[idx]
    run_layer(layer, dynamic=True, static_threshold=5.5)


# ---- config 4: LSTM gate GEMMs, 5-bit weights -------------------------------------------------

@pytest.mark.parametrize("idx", range(2))
def test_config4(idx):
    layer = wl.config(4)[idx]
    run_layer(layer, dynamic=True, static_threshold=None)


# ---- config 5: ResNet-50-shaped sweep, OCS then clip, 4-bit weights ------------------------------

def _unique(layers):
    seen = {}
    for l in layers:
        seen.setdefault((l.M, l.C, l.g, l.N), l)
    return list(seen.values())


def test_config5_weight_path_all_53_layers():
    for layer in wl.config(5, batch=1):
        W = wl.weights(layer)
        for clip in layer.clip_ratios:
            check_weight_path(layer, W, clip)


@pytest.mark.parametrize("idx", range(20))
def test_config5_forward_batch32(idx):
    layer = _unique(wl.config(5, batch=32))[idx]
    run_layer(layer, clips=(0.9,), dynamic=False, static_threshold=5.0)


# The configuration itself: every distinct layer shape at batch 256, the full-size launch the
# benchmark times, static activation grid; the oracle recomputes the first and last 256 rows and
# 4096 seeded random complete rows (codes, accumulators, outputs).  On the two largest activation
# tensors (1.9 GB each), on a narrow-row shape and on the one shape above the MFMA ridge the
# per-batch grid runs as well: max|X| over the whole tensor and every code of the layer against
# the oracle's.
CONFIG5_DYNAMIC = ("stem_7x7", "s1b0_3x3", "s1b0_1x1a", "s4b0_3x3")


@pytest.mark.parametrize("idx", range(20))
def test_config5_forward_batch256(idx):
    layer = _unique(wl.config(5, batch=256))[idx]
    run_layer(layer, clips=(0.8,), dynamic=layer.name in CONFIG5_DYNAMIC, static_threshold=5.0)


# ---- quantization-aware weight split (Sec. 3.3) on the configs' layers ---------------------------

def _check_qa_weights(layer, W, clip):
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, clip_ratio_w=clip)
    L.prepare_weights(dev(W), qa=True)
    exp = ref.split_weights_qa(W, layer.C, layer.g, L.s, layer.bits_w, clip_ratio=clip, ldq=L.ldq)
    assert np.array_equal(host(L.split_src)[:L.s], exp["split_src"])
    assert np.array_equal(host(L.chan_src), exp["chan_src"])
    assert np.array_equal(host(L.chan_depth), exp["chan_depth"])
    assert np.array_equal(host(L.chan_path).view(np.uint32), exp["chan_path"])
    assert np.array_equal(host(L.scale_w), exp["scale"])
    assert np.array_equal(host(L.Wq), exp["q"])
    return L, exp


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_qa_weights_on_configs(cfg):
    for layer in wl.config(cfg):         # config 3: every expand ratio
        _check_qa_weights(layer, wl.weights(layer), layer.clip_ratios[-1])


def test_qa_weights_config5_all_shapes():
    for layer in _unique(wl.config(5)):
        _check_qa_weights(layer, wl.weights(layer), 0.9)


def test_qa_forward_config1_and_lstm_gate():
    for layer in (wl.config(1)[0], wl.shrink(wl.config(4)[0], 256)):
        W, X = wl.weights(layer), wl.activations(layer)
        L, exp = _check_qa_weights(layer, W, 1.0)
        acc = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
        Y = L.forward(dev(X), acc_out=acc)
        Xq_ref, sx_ref, _ = ref.split_act(X, layer.C, layer.g, exp["chan_src"], None, L.s, layer.bits_x,
                                          ldq=L.ldq)
        acc_ref, y_ref = ref.qgemm(Xq_ref, exp["q"], L.Ke, sx_ref[1], exp["scale"][1])
        assert np.array_equal(host(L.Xq[:layer.M]), Xq_ref)
        assert np.array_equal(host(acc), acc_ref)
        assert_y_close(host(Y), y_ref)


# ---- config 2's convolution given un-lowered: lowering inside the kernel, full size ---------------

def test_config2_as_convolution_full_size():
    from paper_1901_09504_amd.layer import ExpandedConv
    (layer,) = wl.config(2)
    Bn, H, Wd_, Cn, N = 64, 14, 14, layer.C, layer.N
    W = wl.weights(layer)
    rng = np.random.default_rng(layer.seed + 7)
    A = np.abs(rng.standard_normal((Bn, H, Wd_, Cn))).astype(np.float32)      # post-ReLU half-normal
    L = ExpandedConv(N, Cn, 3, 3, 1, 1, layer.r, layer.bits_w, layer.bits_x)
    L.prepare_weights(dev(W))
    M = Bn * H * Wd_
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    Y = L.forward(dev(A), acc_out=acc)
    sp = ref.split_weights(W, Cn, 9, L.s)
    Wq_ref, sw_ref = ref.quantize(sp["T_out"], layer.bits_w, ldq=L.w.ldq)
    Aq_ref, sx_ref, _ = ref.split_act(A.reshape(-1, Cn), Cn, 1, sp["chan_src"], None, L.s, layer.bits_x)
    assert np.array_equal(host(L.scale_x), sx_ref) and np.array_equal(host(L.w.scale_w), sw_ref)
    assert np.array_equal(host(L.Aq)[:, :L.E], Aq_ref)
    Xq = np.zeros((M, L.w.ldq), dtype=np.int8)
    Xq[:, :L.E * 9] = ref.im2col(Aq_ref.reshape(Bn, H, Wd_, L.E), 3, 3, 1, 1)
    acc_ref, y_ref = ref.qgemm(Xq, Wq_ref, L.E * 9, sx_ref[1], sw_ref[1])
    assert np.array_equal(host(acc), acc_ref)
    assert_y_close(host(Y), y_ref)
    Y1 = Y.clone()
    assert torch.equal(Y1, L.forward(dev(A)))           # the timed configuration stores no accumulators


# ---- one bottleneck of config 5 at batch 256 as a chain: codes from layer to layer ---------------------

def test_config5_bottleneck_as_a_chain_batch256():
    """The second bottleneck of stage 2 (512 -> 128 1x1, 128 -> 128 3x3, 128 -> 512 1x1 at 28 x 28, batch
    256) with its convolutions given un-lowered and the activations handed on as codes (ReLU, the next
    layer's static grid and duplicated channels): every code tensor between the layers, the last
    layer's accumulators and its outputs, all 200704 rows, against the oracle's chain (split+quantize,
    im2col of the codes, integer GEMM, re-quantization, layer by layer)."""
    from paper_1901_09504_amd.layer import ConvChain
    layers = {l.name: l for l in wl.config(5)}
    la, lb, lc = layers["s2b1_1x1a"], layers["s2b1_3x3"], layers["s2b1_1x1b"]
    Bn, H, Wd_ = 256, 28, 28
    P = Bn * H * Wd_
    assert la.M == P and la.C == 512 and lb.C == 128 and lb.g == 9 and lc.N == 512
    Ws = [wl.weights(la), wl.weights(lb), wl.weights(lc)]
    A = _activations(la)                                   # [P, 512] = the block's input, NHWC
    chain = ConvChain(la.C, [(la.N, 1, 1, 0), (lb.N, 3, 1, 1), (lc.N, 1, 1, 0)], la.r, la.bits_w, la.bits_x,
                      clip_ratio_w=0.9)
    chain.prepare_weights([dev(w) for w in Ws])
    La, Lb, Lc = chain.layers
    # oracle, layer by layer
    T0 = 5.0
    spa = ref.split_weights(Ws[0], la.C, 1, La.s)
    Wqa, swa = ref.quantize(spa["T_out"], la.bits_w, clip_ratio=0.9)
    Aqa, sxa, _ = ref.split_act(A, la.C, 1, spa["chan_src"], None, La.s, la.bits_x, threshold=T0, ldq=La.ldc)
    acca, ya = ref.qgemm(Aqa, Wqa, La.E, sxa[1], swa[1])
    T1 = float(np.float32(0.6) * np.float32(np.abs(ya).max()))
    del ya
    spb = ref.split_weights(Ws[1], lb.C, 9, Lb.s)
    Wqb, swb = ref.quantize(spb["T_out"], lb.bits_w, clip_ratio=0.9)
    Aqb, sxb = ref.requantize(acca, sxa[1], swa[1], T1, lb.bits_x, spb["chan_src"], Lb.s, relu=True, ldq=Lb.ldc)
    Xb = ref.im2col(Aqb[:, :Lb.E].reshape(Bn, H, Wd_, Lb.E), 3, 3, 1, 1)
    accb, yb = ref.qgemm(Xb, Wqb, Lb.E * 9, sxb[1], swb[1])
    T2 = float(np.float32(0.6) * np.float32(np.abs(yb).max()))
    del yb, Xb
    spc = ref.split_weights(Ws[2], lc.C, 1, Lc.s)
    Wqc, swc = ref.quantize(spc["T_out"], lc.bits_w, clip_ratio=0.9)
    Aqc, sxc = ref.requantize(accb, sxb[1], swb[1], T2, lc.bits_x, spc["chan_src"], Lc.s, relu=True, ldq=Lc.ldc)
    accc, yc = ref.qgemm(Aqc, Wqc, Lc.E, sxc[1], swc[1])
    assert (Aqb != 0).mean() > 0.2 and (Aqc != 0).mean() > 0.2      # the grids span the activations
    # GPU
    thr = [torch.tensor([t], dtype=torch.float32, device="cuda") for t in (T0, T1, T2)]
    for L in (La, Lb, Lc):
        L.ensure_input(P)
        L.Aq.fill_(77)                                     # every byte, pad columns included, is the call's to write
    acc = torch.empty((P, lc.N), dtype=torch.int32, device="cuda")
    Y = chain.forward(dev(A).view(Bn, H, Wd_, la.C), thr, acc_out=acc)
    assert np.array_equal(host(La.scale_x), sxa) and np.array_equal(host(La.Aq), Aqa)
    assert np.array_equal(host(Lb.scale_x), sxb) and np.array_equal(host(Lb.Aq), Aqb)
    assert np.array_equal(host(Lc.scale_x), sxc) and np.array_equal(host(Lc.Aq), Aqc)
    assert np.array_equal(host(acc), accc)
    assert_y_close(host(Y), yc)
    Y1 = Y.clone()
    assert torch.equal(Y1, chain.forward(dev(A).view(Bn, H, Wd_, la.C), thr))   # no accumulator dump: same outputs


# ---- the expanded layer run un-expanded: folded weight codes ------------------------------------

@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_folded_layer_equals_expanded_layer(cfg):
    layers = wl.config(cfg) if cfg != 5 else _unique(wl.config(5))[::3]
    fitted = []
    for layer in layers:
        layer = wl.shrink(layer, 640)
        W, X = wl.weights(layer), wl.activations(layer)
        for qa in (False, True):
            L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x)
            L.prepare_weights(dev(W), qa=qa)
            worst = int(host(L.fold_weights())[0])
            Wf_ref, worst_ref = ref.fold_weights(host(L.Wq), layer.C, layer.g, L.s, host(L.chan_src), ldf=L.ldf)
            assert worst == worst_ref, (layer.name, worst, worst_ref)
            assert np.array_equal(host(L.Wf), Wf_ref)
            if worst > 127:
                # a channel with so many copies that their codes do not add up inside int8 (the
                # LSTM layer's dominant channel: 16 copies at 5 bits): folding is reported unusable
                assert cfg == 4
                continue
            fitted.append(layer.name)
            acc_e = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
            acc_f = torch.empty((layer.M, layer.N), dtype=torch.int32, device="cuda")
            Xd = dev(X)
            Y_e = L.forward(Xd, acc_out=acc_e).clone()
            sx_e = host(L.scale_x).copy()
            Y_f = L.forward_folded(Xd, acc_out=acc_f)
            assert np.array_equal(host(L.scale_x), sx_e)
            assert torch.equal(acc_e, acc_f) and torch.equal(Y_e, Y_f)
    assert fitted or cfg == 4


def test_folding_eight_bit_weights_is_reported_as_not_fitting():
    (layer,) = wl.config(2)
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x)
    L.prepare_weights(dev(wl.weights(layer)))
    worst = int(host(L.fold_weights())[0])
    _, worst_ref = ref.fold_weights(host(L.Wq), layer.C, layer.g, L.s, host(L.chan_src))
    assert worst == worst_ref > 127


# ---- the call chain inside a HIP graph ---------------------------------------------------------------

def test_layer_replays_from_a_hip_graph():
    # the library allocates nothing, never synchronises and keeps its scalars on the device, so
    # the whole chain (weights, per-batch grid, split+quantize, GEMM) can be captured once and
    # replayed; every replay is checked against the eager result on the same input
    layer = wl.shrink(wl.config(2)[0], 1500)
    W = wl.weights(layer)
    L = ExpandedLayer(layer.N, layer.C, layer.g, layer.r, layer.bits_w, layer.bits_x, max_rows=layer.M)
    Wd = dev(W)
    Xd = dev(wl.activations(layer))
    L.prepare_weights(Wd)
    L.forward(Xd)                      # eager warm-up: buffers exist before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.prepare_weights(Wd)
        L.forward(Xd)
    rng = np.random.default_rng(3)
    for rep in range(4):
        X = wl.activations(layer) * np.float32(1.0 + rep)
        X[rng.integers(0, layer.M), rng.integers(0, layer.K)] = 40.0 + rep       # moves the per-batch grid
        Xd.copy_(dev(X))
        graph.replay()
        torch.cuda.synchronize()
        Y_graph, sx_graph, Xq_graph = L.Y[:layer.M].clone(), host(L.scale_x).copy(), L.Xq[:layer.M].clone()
        Y_eager = L.forward(Xd).clone()
        torch.cuda.synchronize()
        assert np.array_equal(sx_graph, host(L.scale_x)) and sx_graph[0] == np.float32(40.0 + rep)
        assert torch.equal(Xq_graph, L.Xq[:layer.M]) and torch.equal(Y_graph, Y_eager)
