"""Seeded synthetic layers shaped like the paper's CNN and LSTM workloads.

This module only draws random inputs and lists layer shapes.  It holds none of the
method's arithmetic (no split budget, no quantization, no channel selection), so the CPU
oracle's tests and the GPU path can both take their inputs from it without sharing any
computation.  The paper evaluated ImageNet CNNs from a public model zoo and a two-layer
LSTM language model (Sec. 5, Sec. 6); neither the datasets nor the trained weights are
used here: only the layer shapes and the qualitative "bell-shaped values with rare
outliers" picture of Sec. 1 are imitated.

Seeds: 190109504 + 1000 * config + index of the layer inside the config.  Activations are
drawn in independent blocks of ROW_BLOCK rows, each block from its own child seed, so a
few rows of a very large layer can be regenerated without materialising the whole tensor.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 190109504
ROW_BLOCK = 1024


@dataclass(frozen=True)
class Layer:
    """One linear layer as a GEMM: Y[M,N] = X[M,C*g] @ W[N,C*g]^T."""
    name: str
    config: int
    index: int
    M: int
    C: int          # input channels
    g: int          # K-columns per channel (1 for FC / 1x1 conv, kh*kw for an im2col'd conv)
    N: int          # output channels
    r: float        # expand ratio
    bits_w: int
    bits_x: int
    w_kind: str
    x_kind: str
    clip_ratios: Tuple[float, ...] = (1.0,)
    count: int = 1  # how many times this shape occurs in the network it comes from

    @property
    def K(self):
        return self.C * self.g

    @property
    def seed(self):
        return BASE_SEED + 1000 * self.config + self.index


def _rng(layer, stream, block=0):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([layer.seed, stream, block])))


def weights(layer: Layer) -> np.ndarray:
    """fp32 weights [N, C*g]; channel c owns columns c*g .. c*g+g-1."""
    rng = _rng(layer, 0)
    N, K = layer.N, layer.K
    kind = layer.w_kind
    if kind == "normal_outliers_0.05_0.005_8":       # N(0, 0.05), 0.5 % of entries x8
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
        mask = rng.random((N, K), dtype=np.float32) < np.float32(0.005)
        W = np.where(mask, W * np.float32(8.0), W)
    elif kind == "normal_outliers_0.02_0.001_10":    # N(0, 0.02), 0.1 % of entries x10
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        mask = rng.random((N, K), dtype=np.float32) < np.float32(0.001)
        W = np.where(mask, W * np.float32(10.0), W)
    elif kind == "laplace_0.02":
        W = rng.laplace(0.0, 0.02, (N, K)).astype(np.float32)
    elif kind == "uniform_0.04_t3rows":               # U(-.04,.04); 1 % of rows heavy-tailed
        W = rng.uniform(-0.04, 0.04, (N, K)).astype(np.float32)
        n_heavy = max(1, N // 100)
        rows = rng.choice(N, size=n_heavy, replace=False)
        W[rows] = (0.04 * rng.standard_t(3.0, (n_heavy, K))).astype(np.float32)
    elif kind == "he_normal":                         # N(0, sqrt(2/K))
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(np.sqrt(2.0 / K))
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(W, dtype=np.float32)


def _act_block(layer: Layer, block: int, rows: int) -> np.ndarray:
    rng = _rng(layer, 1, block)
    K = layer.K
    kind = layer.x_kind
    if kind == "normal_t2_outliers":                  # N(0,1), 1 % replaced by 4 * t(df=2)
        X = rng.standard_normal((rows, K), dtype=np.float32)
        mask = rng.random((rows, K), dtype=np.float32) < np.float32(0.01)
        T = (4.0 * rng.standard_t(2.0, (rows, K))).astype(np.float32)
        X = np.where(mask, T, X)
    elif kind == "halfnormal":                        # post-ReLU look: |N(0,1)|
        X = np.abs(rng.standard_normal((rows, K), dtype=np.float32))
    elif kind == "lstm_xh":                           # [x ; h]: N(0,1) | tanh(N(0,1))
        X = rng.standard_normal((rows, K), dtype=np.float32)
        h = K // 2
        X[:, h:] = np.tanh(X[:, h:])
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(X, dtype=np.float32)


def activations(layer: Layer, row0: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """fp32 activations [rows, C*g] for rows row0 .. row0+rows-1 of the layer's X."""
    if rows is None:
        rows = layer.M - row0
    assert 0 <= row0 and row0 + rows <= layer.M
    out = np.empty((rows, layer.K), dtype=np.float32)
    r = row0
    while r < row0 + rows:
        b = r // ROW_BLOCK
        b0 = b * ROW_BLOCK
        nb = min(ROW_BLOCK, layer.M - b0)
        blk = _act_block(layer, b, nb)
        lo = r - b0
        hi = min(nb, row0 + rows - b0)
        out[r - row0:r - row0 + (hi - lo)] = blk[lo:hi]
        r = b0 + hi
    return out


def activations_into(layer: Layer, out: np.ndarray, threads: int = 8) -> np.ndarray:
    """Fill out[:layer.M] (fp32 [>=M, C*g], e.g. a pinned buffer) with the layer's activations,
    drawing the independent row blocks on several threads."""
    from concurrent.futures import ThreadPoolExecutor

    nblocks = (layer.M + ROW_BLOCK - 1) // ROW_BLOCK

    def fill(b):
        b0 = b * ROW_BLOCK
        nb = min(ROW_BLOCK, layer.M - b0)
        out[b0:b0 + nb] = _act_block(layer, b, nb)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(nblocks)))
    return out


# ---------------------------------------------------------------------------------------
# The five configurations
# ---------------------------------------------------------------------------------------

def config1() -> List[Layer]:
    return [Layer("fc_256x256_b64", 1, 0, M=64, C=256, g=1, N=256, r=0.05, bits_w=8, bits_x=8,
                  w_kind="normal_outliers_0.05_0.005_8", x_kind="normal_t2_outliers")]


def config2() -> List[Layer]:
    return [Layer("conv3x3_256_14x14_b64", 2, 0, M=64 * 14 * 14, C=256, g=9, N=256, r=0.02,
                  bits_w=8, bits_x=8, w_kind="laplace_0.02", x_kind="halfnormal")]


def config3() -> List[Layer]:
    shapes = [("conv1x1_1024_256_14x14_b128", 128 * 14 * 14, 1024, 256),
              ("conv1x1_256_1024_14x14_b128", 128 * 14 * 14, 256, 1024),
              ("conv1x1_2048_512_7x7_b128", 128 * 7 * 7, 2048, 512)]
    out = []
    idx = 0
    for name, M, C, N in shapes:
        for r in (0.01, 0.05, 0.1):
            out.append(Layer(f"{name}_r{r}", 3, idx, M=M, C=C, g=1, N=N, r=r, bits_w=6, bits_x=8,
                             w_kind="normal_outliers_0.02_0.001_10", x_kind="halfnormal"))
            idx += 1
    return out


def config4() -> List[Layer]:
    return [Layer(f"lstm{l}_gates_h1500_b20x35", 4, l, M=700, C=3000, g=1, N=6000, r=0.05,
                  bits_w=5, bits_x=8, w_kind="uniform_0.04_t3rows", x_kind="lstm_xh")
            for l in range(2)]


def resnet50_convs(batch: int) -> List[Tuple[str, int, int, int, int]]:
    """(name, C_in, C_out, kernel, M) for the 53 convolutions of a ResNet-50-shaped network
    on 224x224 inputs: 7x7/2 stem, 3x3/2 max-pool, four stages of [3,4,6,3] bottlenecks of
    widths 64/128/256/512 with 4x expansion, the stride of a stage carried by the 3x3 conv
    of its first block, and a 1x1 projection on the first block of every stage."""
    convs = [("stem_7x7", 3, 64, 7, batch * 112 * 112)]
    size = 56
    c_in = 64
    for stage, (blocks, width) in enumerate(zip((3, 4, 6, 3), (64, 128, 256, 512)), start=1):
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 1) else 1
            out_size = size // stride
            tag = f"s{stage}b{b}"
            convs.append((f"{tag}_1x1a", c_in, width, 1, batch * size * size))
            convs.append((f"{tag}_3x3", width, width, 3, batch * out_size * out_size))
            convs.append((f"{tag}_1x1b", width, 4 * width, 1, batch * out_size * out_size))
            if b == 0:
                convs.append((f"{tag}_proj", c_in, 4 * width, 1, batch * out_size * out_size))
            c_in = 4 * width
            size = out_size
    return convs


def config5(batch: int = 256) -> List[Layer]:
    out = []
    for idx, (name, ci, co, k, M) in enumerate(resnet50_convs(batch)):
        out.append(Layer(name, 5, idx, M=M, C=ci, g=k * k, N=co, r=0.05, bits_w=4, bits_x=8,
                         w_kind="he_normal", x_kind="halfnormal", clip_ratios=(1.0, 0.9, 0.8)))
    return out


def config(n: int, **kw) -> List[Layer]:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[n](**kw)


def shrink(layer: Layer, M: int) -> Layer:
    """The same layer with fewer rows (a prefix of its activation rows)."""
    return replace(layer, M=min(M, layer.M))
