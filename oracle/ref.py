"""ctypes front end of oracle/ocs_ref.c (host numpy arrays in, host numpy arrays out).

Test infrastructure only: the GPU library and its Python binding never import this module.
Argument marshalling only; every arithmetic step is in the C file, which cites the
sections and equations of the paper it follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ocs_ref.c")
_LIB = os.path.join(_HERE, "libocs_ref.so")

MODE_HALVE = 0
MODE_DUP = 1

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC"]


def build(force=False):
    """Compile the oracle with gcc (plain C, no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_num_splits.restype = C.c_int
        _lib.ref_num_splits.argtypes = [C.c_int, C.c_double]
        _lib.ref_get_threads.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def set_threads(n):
    lib().ref_set_threads(C.c_int(int(n)))


def get_threads():
    return int(lib().ref_get_threads())


def num_splits(Cn, r):
    return int(lib().ref_num_splits(int(Cn), float(r)))


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with code {rc}")


def split_weights(T, Cn, g, s, mode=MODE_HALVE, split_src=None):
    """Literal one-split-at-a-time OCS on T [rows, C*g].

    Returns dict(split_src, chan_src, chan_depth, T_out [rows,(C+s)*g], max)."""
    T = np.ascontiguousarray(T, dtype=np.float32)
    rows = T.shape[0]
    assert T.shape[1] == Cn * g
    if mode == MODE_DUP:
        ss = np.ascontiguousarray(split_src, dtype=np.int32).copy()
        assert ss.shape[0] == s
    else:
        ss = np.zeros(max(s, 1), dtype=np.int32)
    cs = np.zeros(Cn + s, dtype=np.int32)
    cd = np.zeros(Cn + s, dtype=np.int32)
    out = np.zeros((rows, (Cn + s) * g), dtype=np.float32)
    mx = np.zeros(1, dtype=np.float32)
    rc = lib().ref_split_weights(
        _p(T, C.c_float), C.c_int64(rows), C.c_int(Cn), C.c_int(g), C.c_int64(T.shape[1]),
        C.c_int(s), C.c_int(mode), _p(ss, C.c_int32), _p(cs, C.c_int32), _p(cd, C.c_int32),
        _p(out, C.c_float), C.c_int64(out.shape[1]), _p(mx, C.c_float))
    _check(rc, "ref_split_weights")
    return dict(split_src=ss[:s], chan_src=cs, chan_depth=cd, T_out=out, max=float(mx[0]))


def split_weights_qa(T, Cn, g, s, bits, clip_ratio=1.0, ldq=None):
    """Sec. 3.3: quantization-aware split of T [rows, C*g], then codes by floor(x + 1/2).

    Returns dict(split_src, chan_src, chan_depth, chan_path, T_out, q [rows, ldq], scale)."""
    T = np.ascontiguousarray(T, dtype=np.float32)
    rows = T.shape[0]
    assert T.shape[1] == Cn * g
    Ke = (Cn + s) * g
    ldq = Ke if ldq is None else int(ldq)
    ss = np.zeros(max(s, 1), dtype=np.int32)
    cs = np.zeros(Cn + s, dtype=np.int32)
    cd = np.zeros(Cn + s, dtype=np.int32)
    cp = np.zeros(Cn + s, dtype=np.uint32)
    out = np.zeros((rows, Ke), dtype=np.float32)
    q = np.full((rows, ldq), 99, dtype=np.int8)
    sc = np.zeros(2, dtype=np.float32)
    rc = lib().ref_split_weights_qa(
        _p(T, C.c_float), C.c_int64(rows), C.c_int(Cn), C.c_int(g), C.c_int64(T.shape[1]),
        C.c_int(s), C.c_int(bits), C.c_float(clip_ratio), _p(ss, C.c_int32), _p(cs, C.c_int32),
        _p(cd, C.c_int32), _p(cp, C.c_uint32), _p(out, C.c_float), C.c_int64(Ke),
        _p(q, C.c_int8), C.c_int64(ldq), _p(sc, C.c_float))
    _check(rc, "ref_split_weights_qa")
    return dict(split_src=ss[:s], chan_src=cs, chan_depth=cd, chan_path=cp, T_out=out, q=q, scale=sc)


def mse_clip(x, bits, n_bins=2048, n_cand=512):
    """Sec. 4.1: threshold of least histogram MSE.  Returns dict(threshold, max, hist, mse)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, cols = x.shape
    hist = np.zeros(n_bins, dtype=np.uint64)
    mse = np.zeros(n_cand, dtype=np.float64)
    out = np.zeros(2, dtype=np.float32)
    rc = lib().ref_mse_clip(_p(x, C.c_float), C.c_int64(rows), C.c_int64(cols), C.c_int64(cols),
                            C.c_int(bits), C.c_int(n_bins), C.c_int(n_cand), _p(hist, C.c_uint64),
                            _p(mse, C.c_double), _p(out, C.c_float))
    _check(rc, "ref_mse_clip")
    return dict(threshold=out[0], max=out[1], hist=hist, mse=mse)


def conv_out_size(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


def im2col(A, kh, kw, stride=1, pad=0):
    """The lowering of a convolution to the GEMM of Eq. 2, written out: A [B, H, W, C] (any
    dtype) -> X [B*Ho*Wo, C*kh*kw] with X[(b, yo, xo), c*kh*kw + ky*kw + kx] =
    A[b, yo*stride + ky - pad, xo*stride + kx - pad, c], zero outside the image.  Column order
    matches a [N, C, kh, kw] weight reshaped to [N, C*kh*kw] (channel c owns kh*kw columns)."""
    A = np.asarray(A)
    Bn, H, W, Cn = A.shape
    Ho, Wo = conv_out_size(H, kh, stride, pad), conv_out_size(W, kw, stride, pad)
    X = np.zeros((Bn, Ho, Wo, Cn, kh * kw), dtype=A.dtype)
    for ky in range(kh):
        for kx in range(kw):
            for yo in range(Ho):
                iy = yo * stride + ky - pad
                if iy < 0 or iy >= H:
                    continue
                for xo in range(Wo):
                    ix = xo * stride + kx - pad
                    if 0 <= ix < W:
                        X[:, yo, xo, :, ky * kw + kx] = A[:, iy, ix, :]
    return X.reshape(Bn * Ho * Wo, Cn * kh * kw)


def quantize(x, bits, threshold=None, clip_ratio=1.0, ldq=None):
    """Eq. 1 (+ clip).  Returns (codes [rows, ldq] int8, scale float32[2] = {T, step})."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, cols = x.shape
    ldq = cols if ldq is None else int(ldq)
    q = np.full((rows, ldq), 99, dtype=np.int8)
    sc = np.zeros(2, dtype=np.float32)
    th = None if threshold is None else np.array([threshold], dtype=np.float32)
    rc = lib().ref_quantize(
        _p(x, C.c_float), C.c_int64(rows), C.c_int64(cols), C.c_int64(cols), C.c_int(bits),
        _p(th, C.c_float), C.c_float(clip_ratio), _p(q, C.c_int8), C.c_int64(ldq),
        _p(sc, C.c_float))
    _check(rc, "ref_quantize")
    return q, sc


def split_act(X, Cn, g, chan_src, chan_depth, s, bits, threshold=None, clip_ratio=1.0,
              ldq=None, want_f32=False):
    """Activation side of Eq. 3 (chan_depth None) / Eq. 4, then Eq. 1.

    Returns (codes [M, ldq] int8, scale float32[2], expanded fp32 activations or None)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    M = X.shape[0]
    assert X.shape[1] == Cn * g
    Ke = (Cn + s) * g
    ldq = Ke if ldq is None else int(ldq)
    cs = None if chan_src is None else np.ascontiguousarray(chan_src, dtype=np.int32)
    cd = None if chan_depth is None else np.ascontiguousarray(chan_depth, dtype=np.int32)
    q = np.full((M, ldq), 99, dtype=np.int8)
    sc = np.zeros(2, dtype=np.float32)
    th = None if threshold is None else np.array([threshold], dtype=np.float32)
    Xf = np.zeros((M, Ke), dtype=np.float32) if want_f32 else None
    rc = lib().ref_split_act(
        _p(X, C.c_float), C.c_int64(M), C.c_int(Cn), C.c_int(g), C.c_int64(X.shape[1]),
        _p(cs, C.c_int32), _p(cd, C.c_int32), C.c_int(s), C.c_int(bits), _p(th, C.c_float),
        C.c_float(clip_ratio), _p(q, C.c_int8), C.c_int64(ldq), _p(sc, C.c_float),
        _p(Xf, C.c_float), C.c_int64(Ke))
    _check(rc, "ref_split_act")
    return q, sc, Xf


def split_act_qa(X, Cn, g, split_src, s, bits, T, ldq=None, want_f32=False):
    """Sec. 3.3 on the activations (Eq. 4 with the QA pair).  Returns (codes, scale, Xf or None)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    M = X.shape[0]
    Ke = (Cn + s) * g
    ldq = Ke if ldq is None else int(ldq)
    q = np.full((M, ldq), 99, dtype=np.int8)
    sc = np.zeros(2, dtype=np.float32)
    ss = np.ascontiguousarray(split_src, dtype=np.int32) if s > 0 else None
    Xf = np.zeros((M, Ke), dtype=np.float32) if want_f32 else None
    rc = lib().ref_split_act_qa(_p(X, C.c_float), C.c_int64(M), C.c_int(Cn), C.c_int(g), C.c_int64(X.shape[1]),
                                _p(ss, C.c_int32), C.c_int(s), C.c_int(bits), C.c_float(T), _p(q, C.c_int8),
                                C.c_int64(ldq), _p(sc, C.c_float), _p(Xf, C.c_float), C.c_int64(Ke))
    _check(rc, "ref_split_act_qa")
    return q, sc, Xf


def qgemm(Xq, Wq, Kexp, step_x, step_w, want_acc=True, want_y=True):
    """Eq. 2 on codes.  Returns (acc int32 [M,N] or None, Y float64 [M,N] or None)."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    M, N = Xq.shape[0], Wq.shape[0]
    acc = np.zeros((M, N), dtype=np.int32) if want_acc else None
    Y = np.zeros((M, N), dtype=np.float64) if want_y else None
    rc = lib().ref_qgemm(
        _p(Xq, C.c_int8), C.c_int64(Xq.shape[1]), _p(Wq, C.c_int8), C.c_int64(Wq.shape[1]),
        C.c_int64(M), C.c_int64(N), C.c_int64(Kexp), C.c_float(step_x), C.c_float(step_w),
        _p(acc, C.c_int32), C.c_int64(N), _p(Y, C.c_double), C.c_int64(N))
    _check(rc, "ref_qgemm")
    return acc, Y


def requantize(acc, step_x, step_w, T_next, bits_next, chan_src_next=None, s_next=0, relu=False, ldq=None):
    """The layer's output as the next layer's codes (static grid).  Returns (codes, scale)."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    ldq = N + s_next if ldq is None else int(ldq)
    q = np.full((M, ldq), 99, dtype=np.int8)
    sc = np.zeros(2, dtype=np.float32)
    cs = None if chan_src_next is None else np.ascontiguousarray(chan_src_next, dtype=np.int32)
    rc = lib().ref_requantize(_p(acc, C.c_int32), C.c_int64(N), C.c_int64(M), C.c_int64(N),
                              C.c_float(step_x), C.c_float(step_w), C.c_int(1 if relu else 0),
                              C.c_int(bits_next), C.c_float(T_next), _p(cs, C.c_int32), C.c_int(s_next),
                              _p(q, C.c_int8), C.c_int64(ldq), _p(sc, C.c_float))
    _check(rc, "ref_requantize")
    return q, sc


def fold_weights(Wq, Cn, g, s, chan_src, ldf=None):
    """Weight codes of the expanded layer folded back onto the C original channels.
    Returns (Wf [N, ldf] int8, largest |folded code|)."""
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    N, ldq = Wq.shape
    ldf = Cn * g if ldf is None else int(ldf)
    Wf = np.full((N, ldf), 99, dtype=np.int8)
    mx = np.zeros(1, dtype=np.int32)
    cs = None if chan_src is None else np.ascontiguousarray(chan_src, dtype=np.int32)
    rc = lib().ref_fold_weights(_p(Wq, C.c_int8), C.c_int64(ldq), C.c_int64(N), C.c_int(Cn), C.c_int(g),
                                C.c_int(s), _p(cs, C.c_int32), _p(Wf, C.c_int8), C.c_int64(ldf),
                                _p(mx, C.c_int32))
    _check(rc, "ref_fold_weights")
    return Wf, int(mx[0])


def layer_f64(X, W):
    """Eq. 2 on real operands in fp64: Y = X @ W.T."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = X.shape
    N = W.shape[0]
    assert W.shape[1] == K
    Y = np.zeros((M, N), dtype=np.float64)
    rc = lib().ref_layer_f64(
        _p(X, C.c_float), C.c_int64(K), _p(W, C.c_float), C.c_int64(K), C.c_int64(M),
        C.c_int64(N), C.c_int64(K), _p(Y, C.c_double), C.c_int64(N))
    _check(rc, "ref_layer_f64")
    return Y
