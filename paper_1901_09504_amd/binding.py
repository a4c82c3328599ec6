"""Thin Python binding of libocs.so (ctypes): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/ocs.h;
PyTorch supplies device memory and the stream, nothing else.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libocs.so")

KALIGN = 64
MODE_HALVE = 0
MODE_DUP = 1
MAX_EXPANDED_CHANNELS = 8000


class OcsError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        msg = lib().ocs_strerror(code).decode()
        hip = lib().ocs_last_hip_error().decode()
        super().__init__(f"{what}: {msg} (code {code})" + (f" [{hip}]" if code == -8 and hip else ""))


_lib = None
_vp, _i64, _i32, _f32, _sz = C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_size_t


def lib():
    """Load libocs.so (built in-tree by paper_1901_09504_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_1901_09504_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    L.ocs_strerror.restype = C.c_char_p
    L.ocs_strerror.argtypes = [_i32]
    L.ocs_last_hip_error.restype = C.c_char_p
    L.ocs_last_hip_error.argtypes = []
    L.ocs_num_splits.restype = _i32
    L.ocs_num_splits.argtypes = [_i32, C.c_double]
    L.ocs_padded_cols.restype = _i64
    L.ocs_padded_cols.argtypes = [_i64]
    L.ocs_conv_weight_cols.restype = _i64
    L.ocs_conv_weight_cols.argtypes = [C.c_int, _i64]
    L.ocs_padded_channels.restype = _i64
    L.ocs_padded_channels.argtypes = [_i64]
    L.ocs_workspace_bytes.restype = _sz
    L.ocs_workspace_bytes.argtypes = [_i64, _i64]
    L.ocs_select_channels.restype = _i32
    L.ocs_select_channels.argtypes = [_vp, _i64, _i32, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ocs_split_weights.restype = _i32
    L.ocs_split_weights.argtypes = [_vp, _i64, _i32, _i32, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _i64,
                                    _vp, _i32, _f32, _vp, _i64, _vp, _vp, _sz, _vp]
    L.ocs_split_weights_qa.restype = _i32
    L.ocs_split_weights_qa.argtypes = [_vp, _i64, _i32, _i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _i64,
                                       _i32, _f32, _vp, _i64, _vp, _vp, _sz, _vp]
    L.ocs_mse_clip_threshold.restype = _i32
    L.ocs_mse_clip_threshold.argtypes = [_vp, _i64, _i64, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ocs_conv_weights_tap_major.restype = _i32
    L.ocs_conv_weights_tap_major.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _i64, _vp]
    L.ocs_qconv.restype = _i32
    L.ocs_qconv.argtypes = [_vp, _i64, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _i64, _i32,
                            _i32, _vp, _vp, _vp, _i64, _vp, _i64, _vp]
    L.ocs_qgemm_requant.restype = _i32
    L.ocs_qgemm_requant.argtypes = [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _vp, _vp, _i32, _vp,
                                    _i32, _vp, _i32, _vp, _i64, _vp, _vp, _i64, _vp]
    L.ocs_qconv_requant.restype = _i32
    L.ocs_qconv_requant.argtypes = [_vp, _i64, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _i64, _i32,
                                    _i32, _vp, _vp, _i32, _vp, _i32, _vp, _i32, _vp, _i64, _vp, _vp, _i64, _vp]
    L.ocs_fold_weights.restype = _i32
    L.ocs_fold_weights.argtypes = [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp, _i64, _vp, _vp]
    L.ocs_split_act_qa.restype = _i32
    L.ocs_split_act_qa.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _i64,
                                   _vp, _vp]
    L.ocs_duplicate_weight_codes.restype = _i32
    L.ocs_duplicate_weight_codes.argtypes = [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp]
    L.ocs_quantize.restype = _i32
    L.ocs_quantize.argtypes = [_vp, _i64, _i64, _i64, _i32, _vp, _f32, _vp, _i64, _vp, _vp, _sz, _vp]
    L.ocs_split_act.restype = _i32
    L.ocs_split_act.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _vp, _i32, _i32, _vp, _f32, _vp, _i64,
                                _vp, _vp, _sz, _vp]
    L.ocs_split_act_static.restype = _i32
    L.ocs_split_act_static.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _vp, _i32, _i32, _vp, _f32, _vp, _i64,
                                       _vp, _vp]
    L.ocs_act_threshold.restype = _i32
    L.ocs_act_threshold.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _vp, _i32, _i32, _f32, _vp, _vp, _sz, _vp]
    L.ocs_qgemm.restype = _i32
    L.ocs_qgemm.argtypes = [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _vp, _vp, _vp, _i64, _vp,
                            _i64, _vp, _sz, _vp]
    L.ocs_qgemm_split_k_workspace_bytes.restype = _sz
    L.ocs_qgemm_split_k_workspace_bytes.argtypes = [_i64, _i64, _i64, _i32]
    L.ocs_qgemm_split_k.restype = _i32
    L.ocs_qgemm_split_k.argtypes = [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _i32, _i32, _vp, _vp, _vp, _i64, _vp,
                                    _i64, _i32, _vp, _sz, _vp]
    L.ocs_split_act_qgemm_fits.restype = _i32
    L.ocs_split_act_qgemm_fits.argtypes = [_i64, _i32, _i32, _i32, _i64, _i64]
    L.ocs_split_act_qgemm_pays.restype = _i32
    L.ocs_split_act_qgemm_pays.argtypes = [_i64, _i32, _i32, _i32, _i64, _i64]
    L.ocs_split_act_qgemm.restype = _i32
    L.ocs_split_act_qgemm.argtypes = [_vp, _i64, _i32, _i32, _i64, _vp, _i32, _i32, _vp, _vp, _i64, _i64, _i32, _vp,
                                      _vp, _vp, _i64, _vp, _i64, _vp]
    L.ocs_time_next.restype = _i32
    L.ocs_time_next.argtypes = [_i32, _vp, _vp]
    L.ocs_calib_copy.restype = _i32
    L.ocs_calib_copy.argtypes = [_vp, _vp, _sz, _i32, _vp]
    L.ocs_calib_pack.restype = _i32
    L.ocs_calib_pack.argtypes = [_vp, _vp, _sz, _i32, _vp]
    L.ocs_calib_read.restype = _i32
    L.ocs_calib_read.argtypes = [_vp, _sz, _i32, _i32, _vp, _vp]
    L.ocs_calib_fill.restype = _i32
    L.ocs_calib_fill.argtypes = [_vp, _sz, _i32, _i32, _i32, _vp]
    L.ocs_calib_mfma.restype = _i32
    L.ocs_calib_mfma.argtypes = [_vp, _i32, _i32, _vp, _vp]
    L.ocs_tune.restype = _i32
    L.ocs_tune.argtypes = [C.c_char_p, _i32]
    _lib = L
    return L


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ws(workspace):
    if workspace is None:
        return None, 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _check(rc, what):
    if rc != 0:
        raise OcsError(rc, what)


# ---- host-only helpers ----------------------------------------------------------------------

def ocs_num_splits(Cn, r):
    return int(lib().ocs_num_splits(int(Cn), float(r)))


def ocs_padded_cols(cols):
    return int(lib().ocs_padded_cols(int(cols)))


def ocs_conv_weight_cols(g, ldc):
    return int(lib().ocs_conv_weight_cols(int(g), int(ldc)))


def ocs_padded_channels(channels):
    return int(lib().ocs_padded_channels(int(channels)))


def ocs_workspace_bytes(rows, cols):
    return int(lib().ocs_workspace_bytes(int(rows), int(cols)))


def ocs_qgemm_split_k_workspace_bytes(M, N, Kexp, parts):
    return int(lib().ocs_qgemm_split_k_workspace_bytes(int(M), int(N), int(Kexp), int(parts)))


def ocs_tune(key, value):
    _check(lib().ocs_tune(key.encode(), int(value)), "ocs_tune")


TIME_SPLIT_QUANTIZE = 1
TIME_GEMM = 2
TIME_ABSMAX = 3


def ocs_time_next(family, start_event, stop_event):
    """start_event / stop_event: torch.cuda.Event(enable_timing=True) already recorded once
    (so that their handles exist), or raw hipEvent_t values."""
    a = getattr(start_event, "cuda_event", start_event)
    b = getattr(stop_event, "cuda_event", stop_event)
    _check(lib().ocs_time_next(int(family), C.c_void_p(a), C.c_void_p(b)), "ocs_time_next")


def ocs_calib_copy(src, dst, nbytes, workgroups=0, stream=None):
    _check(lib().ocs_calib_copy(_ptr(src), _ptr(dst), int(nbytes), int(workgroups), _stream(stream)),
           "ocs_calib_copy")


def ocs_calib_pack(src, dst, nbytes, workgroups=0, stream=None):
    _check(lib().ocs_calib_pack(_ptr(src), _ptr(dst), int(nbytes), int(workgroups), _stream(stream)),
           "ocs_calib_pack")


def ocs_calib_read(src, nbytes, passes, workgroups, sink, stream=None):
    _check(lib().ocs_calib_read(_ptr(src), int(nbytes), int(passes), int(workgroups), _ptr(sink),
                                _stream(stream)), "ocs_calib_read")


def ocs_calib_fill(dst, nbytes, value, nontemporal=0, workgroups=0, stream=None):
    _check(lib().ocs_calib_fill(_ptr(dst), int(nbytes), int(value), int(nontemporal), int(workgroups),
                                _stream(stream)), "ocs_calib_fill")


def ocs_calib_mfma(operands, iters, workgroups, sink, stream=None):
    _check(lib().ocs_calib_mfma(_ptr(operands), int(iters), int(workgroups), _ptr(sink), _stream(stream)),
           "ocs_calib_mfma")


def alloc_workspace(rows, cols, device="cuda"):
    """A device buffer large enough for any call on a [rows, cols] fp32 tensor."""
    return torch.empty(max(256, ocs_workspace_bytes(rows, cols)), dtype=torch.uint8, device=device)


# ---- device calls (same names and argument order as the C ABI) ------------------------------

def ocs_select_channels(T, rows, Cn, g, ld, num_splits, split_src, chan_src, chan_depth, max_out,
                        workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_select_channels(_ptr(T), rows, Cn, g, ld, num_splits, _ptr(split_src),
                                     _ptr(chan_src), _ptr(chan_depth), _ptr(max_out), w, wb,
                                     _stream(stream)), "ocs_select_channels")


def ocs_split_weights(W, N, Cn, g, ldw, num_splits, mode, split_src, chan_src, chan_depth, W_out, ldo,
                      wmax_out, bits, clip_ratio, Wq, ldq, scale_w_out, workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_split_weights(_ptr(W), N, Cn, g, ldw, num_splits, mode, _ptr(split_src),
                                   _ptr(chan_src), _ptr(chan_depth), _ptr(W_out), ldo,
                                   _ptr(wmax_out), bits, clip_ratio, _ptr(Wq), ldq,
                                   _ptr(scale_w_out), w, wb, _stream(stream)), "ocs_split_weights")


def ocs_split_weights_qa(W, N, Cn, g, ldw, num_splits, split_src, chan_src, chan_depth, chan_path,
                         W_out, ldo, bits, clip_ratio, Wq, ldq, scale_w_out, workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_split_weights_qa(_ptr(W), N, Cn, g, ldw, num_splits, _ptr(split_src),
                                      _ptr(chan_src), _ptr(chan_depth), _ptr(chan_path), _ptr(W_out),
                                      ldo, bits, clip_ratio, _ptr(Wq), ldq, _ptr(scale_w_out), w, wb,
                                      _stream(stream)), "ocs_split_weights_qa")


def ocs_mse_clip_threshold(x, rows, cols, ldx, bits, num_bins, num_candidates, threshold_out, hist_out,
                           mse_out, workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_mse_clip_threshold(_ptr(x), rows, cols, ldx, bits, num_bins, num_candidates,
                                        _ptr(threshold_out), _ptr(hist_out), _ptr(mse_out), w, wb,
                                        _stream(stream)), "ocs_mse_clip_threshold")


def ocs_conv_weights_tap_major(Wq, N, C_exp, g, ldq, Wt, ldc, stream=None):
    _check(lib().ocs_conv_weights_tap_major(_ptr(Wq), N, C_exp, g, ldq, _ptr(Wt), ldc, _stream(stream)),
           "ocs_conv_weights_tap_major")


def ocs_qconv(Aq, ldc, Bn, H, W, C_exp, kh, kw, stride, pad, Wt, N, bits_x, bits_w, scale_x, scale_w,
              acc_out, ldacc, Y, ldy, stream=None):
    _check(lib().ocs_qconv(_ptr(Aq), ldc, Bn, H, W, C_exp, kh, kw, stride, pad, _ptr(Wt), N, bits_x,
                           bits_w, _ptr(scale_x), _ptr(scale_w), _ptr(acc_out), ldacc, _ptr(Y), ldy,
                           _stream(stream)), "ocs_qconv")


def ocs_qgemm_requant(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, scale_x, scale_w, relu, next_threshold,
                      next_bits, next_chan_src, next_splits, Yq, ldyq, next_scale_out, acc_out=None, ldacc=0,
                      stream=None):
    _check(lib().ocs_qgemm_requant(_ptr(Xq), ldx, _ptr(Wq), ldw, M, N, Kexp, bits_x, bits_w, _ptr(scale_x),
                                   _ptr(scale_w), int(bool(relu)), _ptr(next_threshold), next_bits,
                                   _ptr(next_chan_src), next_splits, _ptr(Yq), ldyq, _ptr(next_scale_out),
                                   _ptr(acc_out), ldacc, _stream(stream)), "ocs_qgemm_requant")


def ocs_qconv_requant(Aq, ldc, Bn, H, W, C_exp, kh, kw, stride, pad, Wt, N, bits_x, bits_w, scale_x, scale_w,
                      relu, next_threshold, next_bits, next_chan_src, next_splits, Yq, ldyq, next_scale_out,
                      acc_out=None, ldacc=0, stream=None):
    _check(lib().ocs_qconv_requant(_ptr(Aq), ldc, Bn, H, W, C_exp, kh, kw, stride, pad, _ptr(Wt), N, bits_x,
                                   bits_w, _ptr(scale_x), _ptr(scale_w), int(bool(relu)),
                                   _ptr(next_threshold), next_bits, _ptr(next_chan_src), next_splits,
                                   _ptr(Yq), ldyq, _ptr(next_scale_out), _ptr(acc_out), ldacc,
                                   _stream(stream)), "ocs_qconv_requant")


def ocs_duplicate_weight_codes(Wq, ldq, N, Cn, g, num_splits, chan_src, stream=None):
    _check(lib().ocs_duplicate_weight_codes(_ptr(Wq), ldq, N, Cn, g, num_splits, _ptr(chan_src),
                                            _stream(stream)), "ocs_duplicate_weight_codes")


def ocs_fold_weights(Wq, ldq, N, Cn, g, num_splits, chan_src, Wf, ldf, max_abs_out, stream=None):
    _check(lib().ocs_fold_weights(_ptr(Wq), ldq, N, Cn, g, num_splits, _ptr(chan_src), _ptr(Wf), ldf,
                                  _ptr(max_abs_out), _stream(stream)), "ocs_fold_weights")


def ocs_split_act_qa(X, M, Cn, g, ldx, split_src, chan_src, chan_depth, chan_path, num_splits, bits, threshold,
                     Xq, ldq, scale_out, stream=None):
    _check(lib().ocs_split_act_qa(_ptr(X), M, Cn, g, ldx, _ptr(split_src), _ptr(chan_src), _ptr(chan_depth),
                                  _ptr(chan_path), num_splits, bits, _ptr(threshold), _ptr(Xq), ldq,
                                  _ptr(scale_out), _stream(stream)), "ocs_split_act_qa")


def ocs_quantize(x, rows, cols, ldx, bits, threshold, clip_ratio, q, ldq, scale_out, workspace,
                 stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_quantize(_ptr(x), rows, cols, ldx, bits, _ptr(threshold), clip_ratio, _ptr(q),
                              ldq, _ptr(scale_out), w, wb, _stream(stream)), "ocs_quantize")


def ocs_split_act(X, M, Cn, g, ldx, chan_src, chan_depth, num_splits, bits, threshold, clip_ratio, Xq,
                  ldq, scale_out, workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_split_act(_ptr(X), M, Cn, g, ldx, _ptr(chan_src), _ptr(chan_depth), num_splits,
                               bits, _ptr(threshold), clip_ratio, _ptr(Xq), ldq, _ptr(scale_out), w,
                               wb, _stream(stream)), "ocs_split_act")


STATIC_SCRATCH_BYTES = 2 * 1024 * 1024


def ocs_split_act_static(X, M, Cn, g, ldx, chan_src, chan_depth, num_splits, bits, threshold, clip_ratio,
                         Xq, ldq, scale_out, stream=None):
    _check(lib().ocs_split_act_static(_ptr(X), M, Cn, g, ldx, _ptr(chan_src), _ptr(chan_depth),
                                      num_splits, bits, _ptr(threshold), clip_ratio, _ptr(Xq), ldq,
                                      _ptr(scale_out), _stream(stream)), "ocs_split_act_static")


def ocs_act_threshold(X, M, Cn, g, ldx, chan_src, chan_depth, num_splits, bits, clip_ratio, scale_out,
                      workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_act_threshold(_ptr(X), M, Cn, g, ldx, _ptr(chan_src), _ptr(chan_depth),
                                   num_splits, bits, clip_ratio, _ptr(scale_out), w, wb,
                                   _stream(stream)), "ocs_act_threshold")


def ocs_qgemm(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, scale_x, scale_w, acc_out, ldacc, Y, ldy,
              workspace=None, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_qgemm(_ptr(Xq), ldx, _ptr(Wq), ldw, M, N, Kexp, bits_x, bits_w, _ptr(scale_x),
                           _ptr(scale_w), _ptr(acc_out), ldacc, _ptr(Y), ldy, w, wb,
                           _stream(stream)), "ocs_qgemm")


def ocs_split_act_qgemm_fits(M, C, g, num_splits, N, ldx):
    return bool(lib().ocs_split_act_qgemm_fits(int(M), int(C), int(g), int(num_splits), int(N), int(ldx)))


def ocs_split_act_qgemm_pays(M, C, g, num_splits, N, ldx):
    return bool(lib().ocs_split_act_qgemm_pays(int(M), int(C), int(g), int(num_splits), int(N), int(ldx)))


def ocs_split_act_qgemm(X, M, C, g, ldx, chan_src, num_splits, bits_x, threshold, Wq, ldw, N, bits_w, scale_w,
                        scale_x_out, acc_out, ldacc, Y, ldy, stream=None):
    _check(lib().ocs_split_act_qgemm(_ptr(X), M, C, g, ldx, _ptr(chan_src), num_splits, bits_x, _ptr(threshold),
                                     _ptr(Wq), ldw, N, bits_w, _ptr(scale_w), _ptr(scale_x_out), _ptr(acc_out),
                                     ldacc, _ptr(Y), ldy, _stream(stream)), "ocs_split_act_qgemm")


def ocs_qgemm_split_k(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, scale_x, scale_w, acc_out, ldacc, Y, ldy,
                      parts, workspace, stream=None):
    w, wb = _ws(workspace)
    _check(lib().ocs_qgemm_split_k(_ptr(Xq), ldx, _ptr(Wq), ldw, M, N, Kexp, bits_x, bits_w, _ptr(scale_x),
                                   _ptr(scale_w), _ptr(acc_out), ldacc, _ptr(Y), ldy, int(parts), w, wb,
                                   _stream(stream)), "ocs_qgemm_split_k")
