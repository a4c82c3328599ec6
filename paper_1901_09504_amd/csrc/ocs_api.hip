// C ABI of libocs.so: argument validation (host only, before any device work), workspace
// carving, and the launch sequences.  See include/ocs.h for the contract of each call.
#include <string.h>

#include <atomic>
#include <string>

#include "../../include/ocs.h"
#include "ocs_internal.h"

namespace ocs {

Tuning& tuning() {
    static thread_local Tuning t;
    return t;
}

KernelTimer& kernel_timer() {
    static thread_local KernelTimer t;
    return t;
}

static thread_local std::string g_hip_error;

static int hip_fail(hipError_t e) {
    g_hip_error = hipGetErrorString(e);
    return OCS_E_HIP;
}

constexpr int kStaticScratchDevices = 64;   // devices a process can see

static bool bits_ok(int bits) { return bits >= 2 && bits <= 8; }
static float qmax_of(int bits) { return (float)((1 << (bits - 1)) - 1); }
// Sec. 4 clips at a fraction of the range; any positive finite factor gives a usable grid
static bool clip_ok(float c) { return c > 0.0f && c <= 3.402823466e+38f; }
static bool aligned(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

static int check_codes(const void* q, int64_t ldq, int64_t cols) {
    if (ldq < cols) return OCS_E_SHAPE;
    if (ldq % OCS_CALIGN != 0 || !aligned(q, 16)) return OCS_E_ALIGN;
    return OCS_OK;
}

static int check_workspace(const void* ws, size_t ws_bytes, int64_t rows, int64_t cols) {
    if (ws == nullptr || ws_bytes < plan_workspace(rows, cols).total) return OCS_E_WORKSPACE;
    if (!aligned(ws, 256)) return OCS_E_ALIGN;
    return OCS_OK;
}

static int check_layer(int64_t rows, int C, int g, int64_t ld, int num_splits) {
    if (rows <= 0 || C <= 0 || g <= 0) return OCS_E_SHAPE;
    if ((int64_t)C * g > (int64_t)1 << 30 || rows > (int64_t)1 << 31) return OCS_E_SHAPE;
    if (ld < (int64_t)C * g) return OCS_E_SHAPE;
    if (num_splits < 0) return OCS_E_SPLITS;
    if ((int64_t)C + num_splits > OCS_MAX_EXPANDED_CHANNELS) return OCS_E_SPLITS;
    return OCS_OK;
}

// Operands of the GEMM: shapes, leading dimensions, alignment, and that the int32 accumulator
// cannot overflow for these bit widths.
static int check_gemm_operands(const void* Xq, int64_t ldx, const void* Wq, int64_t ldw, int64_t M,
                               int64_t N, int64_t Kexp, int bits_x, int bits_w, const void* acc_out,
                               int64_t ldacc) {
    if (M <= 0 || N <= 0 || Kexp <= 0) return OCS_E_SHAPE;
    if (M > (int64_t)1 << 30 || N > (int64_t)1 << 30 || Kexp > (int64_t)1 << 30) return OCS_E_SHAPE;
    const int64_t Kpad = round_up(Kexp, OCS_KALIGN);
    // up to OCS_SHORT_K bytes of K (rounded up to the K-step) the pitch only has to hold the row
    // in whole 16-byte pieces; beyond, it holds whole K-steps
    const bool short_k = Kpad <= OCS_SHORT_K;
    const int64_t need = short_k ? round_up(Kexp, OCS_CALIGN) : Kpad;
    const int64_t unit = short_k ? OCS_CALIGN : OCS_KALIGN;
    if (ldx < need || ldw < need || (acc_out && ldacc < N)) return OCS_E_SHAPE;
    if (ldx % unit != 0 || ldw % unit != 0 || !aligned(Xq, 16) || !aligned(Wq, 16))
        return OCS_E_ALIGN;
    if (!bits_ok(bits_x) || !bits_ok(bits_w)) return OCS_E_BITS;
    const int64_t qx = (1 << (bits_x - 1)) - 1, qw = (1 << (bits_w - 1)) - 1;
    if (Kexp * qx * qw >= (int64_t)1 << 31) return OCS_E_OVERFLOW;
    return OCS_OK;
}

// The same for the convolution whose lowering happens inside the kernel.
static int check_conv_operands(const void* Aq, int64_t ldc, int B, int H, int W, int C_exp, int kh,
                               int kw, int stride, int pad, const void* Wt, int64_t N, int bits_x,
                               int bits_w, const void* acc_out, int64_t ldacc) {
    if (B <= 0 || H <= 0 || W <= 0 || C_exp <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0 ||
        N <= 0 || N > (int64_t)1 << 30)
        return OCS_E_SHAPE;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return OCS_E_SHAPE;
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
    if ((int64_t)B * Ho * Wo > (int64_t)1 << 30 || (int64_t)B * H * W > (int64_t)1 << 31) return OCS_E_SHAPE;
    if (ldc < C_exp || (int64_t)kh * kw * ldc > (int64_t)1 << 30) return OCS_E_SHAPE;
    if (acc_out && ldacc < N) return OCS_E_SHAPE;
    if (ldc % OCS_CALIGN != 0 || !aligned(Aq, 16) || !aligned(Wt, 16)) return OCS_E_ALIGN;
    if (!bits_ok(bits_x) || !bits_ok(bits_w)) return OCS_E_BITS;
    const int64_t qx = (1 << (bits_x - 1)) - 1, qw = (1 << (bits_w - 1)) - 1;
    if ((int64_t)kh * kw * C_exp * qx * qw >= (int64_t)1 << 31) return OCS_E_OVERFLOW;
    return OCS_OK;
}

}  // namespace ocs

using namespace ocs;

extern "C" {

const char* ocs_strerror(int code) {
    switch (code) {
        case OCS_OK: return "ok";
        case OCS_E_NULL: return "a required pointer is NULL";
        case OCS_E_SHAPE: return "bad shape: non-positive or too large dimension, or leading dimension too small";
        case OCS_E_ALIGN: return "misaligned code tensor, leading dimension or workspace";
        case OCS_E_BITS: return "bit width outside 2..8";
        case OCS_E_SPLITS: return "num_splits negative, or C + num_splits above OCS_MAX_EXPANDED_CHANNELS";
        case OCS_E_OVERFLOW: return "Kexp * qmax_x * qmax_w does not fit a 32-bit accumulator";
        case OCS_E_WORKSPACE: return "workspace NULL or smaller than ocs_workspace_bytes()";
        case OCS_E_HIP: return "a HIP call failed (see ocs_last_hip_error)";
        case OCS_E_MODE: return "unknown mode or key";
        case OCS_E_CLIP: return "clip_ratio is not a positive finite number";
        default: return "unknown error code";
    }
}

const char* ocs_last_hip_error(void) { return g_hip_error.c_str(); }

int ocs_num_splits(int C, double r) {
    if (C <= 0 || !(r > 0.0)) return 0;
    double v = r * (double)C;
    int s = (int)v;
    if ((double)s < v) ++s;
    return s;
}

int64_t ocs_padded_cols(int64_t cols) {
    if (cols <= 0) return 0;
    // rows of at most 320 bytes go through the GEMM's whole-K kernel, which streams them once:
    // more padding there is only more bytes (measured: 128-byte rows cost those layers 5-25 %)
    return round_up(cols, OCS_KALIGN) <= OCS_SHORT_K ? round_up(cols, OCS_CALIGN) : round_up(cols, OCS_ROWALIGN);
}

int64_t ocs_conv_weight_cols(int g, int64_t ldc) {
    return (g <= 0 || ldc <= 0) ? 0 : round_up((int64_t)g * ldc, OCS_KALIGN);
}

int64_t ocs_padded_channels(int64_t channels) {
    return channels <= 0 ? 0 : round_up(channels, OCS_CALIGN);
}

size_t ocs_workspace_bytes(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return 0;
    return plan_workspace(rows, cols).total;
}

int ocs_select_channels(const float* T, int64_t rows, int C, int g, int64_t ld, int num_splits,
                        int32_t* split_src, int32_t* chan_src, int32_t* chan_depth,
                        float* max_out, void* workspace, size_t ws_bytes, void* stream) {
    if (!T || !chan_src || !chan_depth || (num_splits > 0 && !split_src)) return OCS_E_NULL;
    int rc = check_layer(rows, C, g, ld, num_splits);
    if (rc) return rc;
    const int64_t K = (int64_t)C * g;
    rc = check_workspace(workspace, ws_bytes, rows, K);
    if (rc) return rc;
    Workspace w = plan_workspace(rows, K);
    char* base = static_cast<char*>(workspace);
    float* colmax = reinterpret_cast<float*>(base + w.colmax_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = launch_colmax(T, rows, K, ld, colmax, partial, st);
    if (e != hipSuccess) return hip_fail(e);
    e = launch_select(colmax, C, g, num_splits, 0, nullptr, split_src, chan_src, chan_depth,
                      max_out, 1.0f, 1.0f, nullptr, st);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_split_weights(const float* W, int64_t N, int C, int g, int64_t ldw, int num_splits,
                      int mode, int32_t* split_src, int32_t* chan_src, int32_t* chan_depth,
                      float* W_out, int64_t ldo, float* wmax_out, int bits, float clip_ratio,
                      int8_t* Wq, int64_t ldq, float* scale_w_out, void* workspace,
                      size_t ws_bytes, void* stream) {
    if (!W || !chan_src || !chan_depth || (num_splits > 0 && !split_src)) return OCS_E_NULL;
    if (Wq && !scale_w_out) return OCS_E_NULL;
    if (mode != OCS_MODE_HALVE && mode != OCS_MODE_DUP) return OCS_E_MODE;
    int rc = check_layer(N, C, g, ldw, num_splits);
    if (rc) return rc;
    const int64_t K = (int64_t)C * g, Ke = (int64_t)(C + num_splits) * g;
    if (W_out && ldo < Ke) return OCS_E_SHAPE;
    if (Wq) {
        rc = check_codes(Wq, ldq, Ke);
        if (rc) return rc;
        if (!bits_ok(bits)) return OCS_E_BITS;
        if (!clip_ok(clip_ratio)) return OCS_E_CLIP;
    }
    rc = check_workspace(workspace, ws_bytes, N, K);
    if (rc) return rc;

    Workspace w = plan_workspace(N, K);
    char* base = static_cast<char*>(workspace);
    float* colmax = reinterpret_cast<float*>(base + w.colmax_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = static_cast<hipStream_t>(stream);

    // W1: channel maxima.  W2: selection (or replay of the given list).  The selector also
    // emits max|W'| and, when codes are wanted, the threshold and step of the weight grid.
    hipError_t e = launch_colmax(W, N, K, ldw, colmax, partial, st);
    if (e != hipSuccess) return hip_fail(e);
    const float qmax = Wq ? qmax_of(bits) : 1.0f;
    if (Wq && !W_out && mode == OCS_MODE_HALVE && select_expand_quantize_fits(C, num_splits, N, ldq)) {
        // few splits, codes only: W2 and W3 as one launch
        e = launch_select_expand_quantize(W, ldw, N, C, g, num_splits, colmax, split_src, chan_src,
                                          chan_depth, wmax_out, clip_ratio, qmax, scale_w_out, Wq,
                                          ldq, st);
        return e == hipSuccess ? OCS_OK : hip_fail(e);
    }
    e = launch_select(colmax, C, g, num_splits, mode, split_src, split_src, chan_src, chan_depth,
                      wmax_out, clip_ratio, qmax, Wq ? scale_w_out : nullptr, st);
    if (e != hipSuccess) return hip_fail(e);

    // W3: materialise, as fp32 and / or straight to codes
    const int halve = mode == OCS_MODE_HALVE;
    if (W_out) {
        e = launch_expand_f32(W, ldw, N, C, g, num_splits, chan_src, chan_depth, halve, W_out,
                              ldo, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (Wq) {
        e = launch_expand_quantize(W, ldw, N, C, g, num_splits, chan_src,
                                   halve ? chan_depth : nullptr, scale_w_out, qmax, Wq, ldq,
                                   nullptr, st, nullptr, 0, 1.0f, /*stepwise=*/halve != 0);
        if (e != hipSuccess) return hip_fail(e);
    }
    return OCS_OK;
}

int ocs_split_weights_qa(const float* W, int64_t N, int C, int g, int64_t ldw, int num_splits,
                         int32_t* split_src, int32_t* chan_src, int32_t* chan_depth,
                         uint32_t* chan_path, float* W_out, int64_t ldo, int bits,
                         float clip_ratio, int8_t* Wq, int64_t ldq, float* scale_w_out,
                         void* workspace, size_t ws_bytes, void* stream) {
    if (!W || !chan_src || !chan_depth || !chan_path || !scale_w_out) return OCS_E_NULL;
    if (num_splits > 0 && !split_src) return OCS_E_NULL;
    if (!W_out && !Wq) return OCS_E_NULL;
    int rc = check_layer(N, C, g, ldw, num_splits);
    if (rc) return rc;
    const int64_t K = (int64_t)C * g, Ke = (int64_t)(C + num_splits) * g;
    if (W_out && ldo < Ke) return OCS_E_SHAPE;
    if (Wq) {
        rc = check_codes(Wq, ldq, Ke);
        if (rc) return rc;
    }
    if (!bits_ok(bits)) return OCS_E_BITS;   // the step depends on the grid even without codes
    if (!clip_ok(clip_ratio)) return OCS_E_CLIP;
    rc = check_workspace(workspace, ws_bytes, N, K);
    if (rc) return rc;

    Workspace w = plan_workspace(N, K);
    char* base = static_cast<char*>(workspace);
    float* colmax = reinterpret_cast<float*>(base + w.colmax_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = static_cast<hipStream_t>(stream);

    // selection and threshold exactly as for plain halving; then the histories; then the members
    hipError_t e = launch_colmax(W, N, K, ldw, colmax, partial, st);
    if (e != hipSuccess) return hip_fail(e);
    const float qmax = qmax_of(bits);
    e = launch_select(colmax, C, g, num_splits, OCS_MODE_HALVE, split_src, split_src, chan_src,
                      chan_depth, nullptr, clip_ratio, qmax, scale_w_out, st);
    if (e != hipSuccess) return hip_fail(e);
    e = launch_qa_paths(split_src, C, num_splits, chan_path, st);
    if (e != hipSuccess) return hip_fail(e);
    e = launch_expand_quantize_qa(W, ldw, N, C, g, num_splits, chan_src, chan_depth, chan_path,
                                  scale_w_out, nullptr, qmax, W_out, ldo, Wq, ldq, st);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_split_act_qa(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* split_src,
                     const int32_t* chan_src, const int32_t* chan_depth, uint32_t* chan_path,
                     int num_splits, int bits, const float* threshold, int8_t* Xq, int64_t ldq,
                     float* scale_out, void* stream) {
    if (!X || !Xq || !scale_out || !threshold || !chan_src || !chan_depth || !chan_path) return OCS_E_NULL;
    if (num_splits > 0 && !split_src) return OCS_E_NULL;
    if (threshold == scale_out) return OCS_E_MODE;
    int rc = check_layer(M, C, g, ldx, num_splits);
    if (rc) return rc;
    rc = check_codes(Xq, ldq, (int64_t)(C + num_splits) * g);
    if (rc) return rc;
    if (!bits_ok(bits)) return OCS_E_BITS;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float qmax = qmax_of(bits);
    hipError_t e = launch_qa_paths(split_src, C, num_splits, chan_path, st);
    if (e != hipSuccess) return hip_fail(e);
    e = launch_expand_quantize_qa(X, ldx, M, C, g, num_splits, chan_src, chan_depth, chan_path, threshold,
                                  scale_out, qmax, nullptr, 0, Xq, ldq, st);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_quantize(const float* x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                 const float* threshold, float clip_ratio, int8_t* q, int64_t ldq,
                 float* scale_out, void* workspace, size_t ws_bytes, void* stream) {
    if (!x || !q || !scale_out) return OCS_E_NULL;
    if (rows <= 0 || cols <= 0 || cols > (int64_t)1 << 30 || rows > (int64_t)1 << 31 || ldx < cols)
        return OCS_E_SHAPE;
    int rc = check_codes(q, ldq, cols);
    if (rc) return rc;
    if (!bits_ok(bits)) return OCS_E_BITS;
    if (!threshold && !clip_ok(clip_ratio)) return OCS_E_CLIP;
    const float qmax = qmax_of(bits);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (threshold == nullptr) {
        rc = check_workspace(workspace, ws_bytes, rows, cols);
        if (rc) return rc;
        Workspace w = plan_workspace(rows, cols);
        char* base = static_cast<char*>(workspace);
        float* colmax = reinterpret_cast<float*>(base + w.colmax_off);
        float* partial = reinterpret_cast<float*>(base + w.partial_off);
        (void)colmax;
        int n = 0;
        e = launch_absmax_partials(x, rows, cols, ldx, partial, &n, st);
        if (e != hipSuccess) return hip_fail(e);
        e = launch_expand_quantize(x, ldx, rows, (int)cols, 1, 0, nullptr, nullptr, nullptr, qmax,
                                   q, ldq, scale_out, st, partial, n, clip_ratio);
    } else {
        e = launch_expand_quantize(x, ldx, rows, (int)cols, 1, 0, nullptr, nullptr, threshold, qmax,
                                   q, ldq, scale_out, st);
    }
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_act_threshold(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* chan_src,
                      const int32_t* chan_depth, int num_splits, int bits, float clip_ratio,
                      float* scale_out, void* workspace, size_t ws_bytes, void* stream) {
    if (!X || !scale_out || (num_splits > 0 && !chan_src)) return OCS_E_NULL;
    int rc = check_layer(M, C, g, ldx, num_splits);
    if (rc) return rc;
    if (!bits_ok(bits)) return OCS_E_BITS;
    if (!clip_ok(clip_ratio)) return OCS_E_CLIP;
    const int64_t K = (int64_t)C * g;
    rc = check_workspace(workspace, ws_bytes, M, K);
    if (rc) return rc;
    // X1: column maxima of X, then the maximum over the expanded channels
    Workspace w = plan_workspace(M, K);
    char* base = static_cast<char*>(workspace);
    float* colmax = reinterpret_cast<float*>(base + w.colmax_off);
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (chan_depth == nullptr) {
        // copies do not change the maximum: max|X| of the whole tensor is enough
        (void)colmax;
        e = launch_absmax_threshold(X, M, K, ldx, partial, clip_ratio, qmax_of(bits), scale_out, st);
        if (e != hipSuccess) return hip_fail(e);
    } else {
        e = launch_colmax(X, M, K, ldx, colmax, partial, st);
        if (e != hipSuccess) return hip_fail(e);
        e = launch_threshold(colmax, C, g, num_splits, chan_src, chan_depth, clip_ratio,
                             qmax_of(bits), scale_out, st);
        if (e != hipSuccess) return hip_fail(e);
    }
    return OCS_OK;
}

int ocs_mse_clip_threshold(const float* x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                           int num_bins, int num_candidates, float* threshold_out,
                           unsigned long long* hist_out, double* mse_out, void* workspace,
                           size_t ws_bytes, void* stream) {
    if (!x || !threshold_out || !hist_out || !mse_out) return OCS_E_NULL;
    if (rows <= 0 || cols <= 0 || cols > (int64_t)1 << 30 || rows > (int64_t)1 << 31 || ldx < cols)
        return OCS_E_SHAPE;
    if (num_bins < 1 || num_bins > 8192 || num_candidates < 1 || num_candidates > 65536)
        return OCS_E_SHAPE;
    if (!bits_ok(bits)) return OCS_E_BITS;
    int rc = check_workspace(workspace, ws_bytes, rows, cols);
    if (rc) return rc;
    Workspace w = plan_workspace(rows, cols);
    char* base = static_cast<char*>(workspace);
    float* colmax = reinterpret_cast<float*>(base + w.colmax_off);   // two floats used: {max, step}
    float* partial = reinterpret_cast<float*>(base + w.partial_off);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float qmax = qmax_of(bits);
    int n = 0;
    hipError_t e = launch_absmax_partials(x, rows, cols, ldx, partial, &n, st);
    if (e != hipSuccess) return hip_fail(e);
    e = launch_mse_clip(x, ldx, rows, cols, partial, n, colmax, num_bins, num_candidates, qmax,
                        hist_out, mse_out, threshold_out, st);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

// Argument checks of ocs_split_act that do not concern the scratch space.
static int check_split_act(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* chan_src,
                           int num_splits, int bits, const float* threshold, float clip_ratio,
                           const int8_t* Xq, int64_t ldq, const float* scale_out) {
    if (!X || !Xq || !scale_out || (num_splits > 0 && !chan_src)) return OCS_E_NULL;
    int rc = check_layer(M, C, g, ldx, num_splits);
    if (rc) return rc;
    rc = check_codes(Xq, ldq, (int64_t)(C + num_splits) * g);
    if (rc) return rc;
    if (!bits_ok(bits)) return OCS_E_BITS;
    if (!threshold && !clip_ok(clip_ratio)) return OCS_E_CLIP;
    return OCS_OK;
}

int ocs_split_act(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* chan_src,
                  const int32_t* chan_depth, int num_splits, int bits, const float* threshold,
                  float clip_ratio, int8_t* Xq, int64_t ldq, float* scale_out, void* workspace,
                  size_t ws_bytes, void* stream) {
    int rc = check_split_act(X, M, C, g, ldx, chan_src, num_splits, bits, threshold, clip_ratio, Xq, ldq,
                             scale_out);
    if (rc) return rc;
    const float qmax = qmax_of(bits);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (threshold == nullptr && chan_depth == nullptr) {
        // X1 + X2 with Eq. 3 (copies are not scaled): the expanded tensor's largest magnitude is
        // X's own.  One pass leaves per-workgroup maxima, the streaming pass folds them itself.
        rc = check_workspace(workspace, ws_bytes, M, (int64_t)C * g);
        if (rc) return rc;
        Workspace w = plan_workspace(M, (int64_t)C * g);
        float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + w.partial_off);
        int n = 0;
        hipError_t e = launch_absmax_partials(X, M, (int64_t)C * g, ldx, partial, &n, st);
        if (e != hipSuccess) return hip_fail(e);
        // From 160 MB on the maxima are folded into one word by a launch of its own: the streaming
        // pass then takes its one-shot form, whose workgroups are far too many and too short to fold
        // a few hundred maxima each (config 5's per-batch pass: 13.4 -> 13.1 ms; on a 116 MB tensor the
        // extra launch costs what the faster pass gains).
        const int64_t cap = (int64_t)(w.total - w.partial_off) / 4;
        if (n > 1 && n < cap && (tuning().max_flat == 2 || M * (int64_t)C * g >= ((int64_t)40 << 20))) {   // (max_flat 2: always, for tests)
            e = launch_fold_max(partial, n, partial + n, st);
            if (e != hipSuccess) return hip_fail(e);
            partial += n;
            n = 1;
        }
        e = launch_expand_quantize(X, ldx, M, C, g, num_splits, chan_src, nullptr, nullptr, qmax, Xq,
                                   ldq, scale_out, st, partial, n, clip_ratio);
        if (e != hipSuccess) return hip_fail(e);
        return OCS_OK;
    }
    if (threshold == nullptr) {
        // X1: the dynamic grid needs max|expanded activations| before the streaming pass
        rc = ocs_act_threshold(X, M, C, g, ldx, chan_src, chan_depth, num_splits, bits, clip_ratio,
                               scale_out, workspace, ws_bytes, stream);
        if (rc) return rc;
        threshold = scale_out;
    }
    // X2: one streaming pass.  When the threshold already lives in scale_out the kernel must
    // not rewrite it while other lanes read it.
    hipError_t e = launch_expand_quantize(X, ldx, M, C, g, num_splits, chan_src, chan_depth,
                                          threshold, qmax, Xq, ldq,
                                          threshold == scale_out ? nullptr : scale_out, st);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

// Scratch space of ocs_split_act_static: one array per GPU, part of the library's device image,
// so nothing is allocated at run time.  In host code the name `scratch` is only a handle for
// hipGetSymbolAddress; the address each device holds its copy at is looked up once per device
// (with that device current) and kept, and only that address is ever handed to a launch.
static __device__ __align__(256) unsigned char scratch[OCS_STATIC_SCRATCH_BYTES];

static int static_scratch(void** out) {
    static std::atomic<void*> addr[kStaticScratchDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kStaticScratchDevices) return hip_fail(hipErrorInvalidDevice);
    void* p = addr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (p == nullptr) return hip_fail(hipErrorInvalidSymbol);
        addr[dev].store(p, std::memory_order_release);   // two threads racing here store the same value
    }
    *out = p;
    return OCS_OK;
}

int ocs_split_act_static(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* chan_src,
                         const int32_t* chan_depth, int num_splits, int bits, const float* threshold,
                         float clip_ratio, int8_t* Xq, int64_t ldq, float* scale_out, void* stream) {
    int rc = check_split_act(X, M, C, g, ldx, chan_src, num_splits, bits, threshold, clip_ratio, Xq, ldq,
                             scale_out);
    if (rc) return rc;
    if (plan_workspace(M, (int64_t)C * g).total > (size_t)OCS_STATIC_SCRATCH_BYTES) return OCS_E_WORKSPACE;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    // Every float of the scratch space that a pass reads was written by the pass before it in this
    // same call (per-workgroup maxima, column maxima): nothing has to start at zero, and what an
    // earlier call left behind is never read.
    return ocs_split_act(X, M, C, g, ldx, chan_src, chan_depth, num_splits, bits, threshold, clip_ratio,
                         Xq, ldq, scale_out, ws, (size_t)OCS_STATIC_SCRATCH_BYTES, stream);
}

int ocs_qgemm(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M, int64_t N,
              int64_t Kexp, int bits_x, int bits_w, const float* scale_x, const float* scale_w,
              int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, void* workspace,
              size_t ws_bytes, void* stream) {
    (void)workspace;
    (void)ws_bytes;
    if (!Xq || !Wq || !scale_x || !scale_w || !Y) return OCS_E_NULL;
    int rc = check_gemm_operands(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, acc_out, ldacc);
    if (rc) return rc;
    if (ldy < N) return OCS_E_SHAPE;
    const int64_t Kpad = round_up(Kexp, OCS_KALIGN);
    hipError_t e = launch_qgemm(Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w, acc_out, ldacc, Y,
                                ldy, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_split_act_qgemm_fits(int64_t M, int C, int g, int num_splits, int64_t N, int64_t ldx) {
    if (M <= 0 || C <= 0 || g <= 0 || num_splits < 0 || N <= 0) return 0;
    if ((int64_t)C * g > (int64_t)1 << 30 || (int64_t)C + num_splits > OCS_MAX_EXPANDED_CHANNELS) return 0;
    return split_act_qgemm_fits(M, C, g, num_splits, N, ldx) ? 1 : 0;
}

int ocs_split_act_qgemm_pays(int64_t M, int C, int g, int num_splits, int64_t N, int64_t ldx) {
    if (!ocs_split_act_qgemm_fits(M, C, g, num_splits, N, ldx)) return 0;
    return split_act_qgemm_pays(M, C, g, num_splits, N, ldx) ? 1 : 0;
}

int ocs_split_act_qgemm(const float* X, int64_t M, int C, int g, int64_t ldx, const int32_t* chan_src,
                        int num_splits, int bits_x, const float* threshold, const int8_t* Wq, int64_t ldw,
                        int64_t N, int bits_w, const float* scale_w, float* scale_x_out, int32_t* acc_out,
                        int64_t ldacc, float* Y, int64_t ldy, void* stream) {
    if (!X || !threshold || !Wq || !scale_w || !Y || (num_splits > 0 && !chan_src)) return OCS_E_NULL;
    int rc = check_layer(M, C, g, ldx, num_splits);
    if (rc) return rc;
    if (N <= 0 || N > (int64_t)1 << 30 || ldy < N || (acc_out && ldacc < N)) return OCS_E_SHAPE;
    const int64_t Kexp = (int64_t)(C + num_splits) * g;
    if (ldw < round_up(Kexp, OCS_CALIGN)) return OCS_E_SHAPE;
    if (ldw % OCS_CALIGN != 0 || !aligned(Wq, 16)) return OCS_E_ALIGN;
    if (!bits_ok(bits_x) || !bits_ok(bits_w)) return OCS_E_BITS;
    const int64_t qx = (1 << (bits_x - 1)) - 1, qw = (1 << (bits_w - 1)) - 1;
    if (Kexp * qx * qw >= (int64_t)1 << 31) return OCS_E_OVERFLOW;
    if (scale_x_out == threshold) return OCS_E_MODE;   // the kernel reads one while writing the other
    if (!split_act_qgemm_fits(M, C, g, num_splits, N, ldx)) return OCS_E_SHAPE;
    hipError_t e = launch_split_act_qgemm(X, ldx, M, C, g, num_splits, chan_src, threshold, qmax_of(bits_x), Wq,
                                          ldw, N, Kexp, scale_w, scale_x_out, acc_out, ldacc, Y, ldy,
                                          static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

size_t ocs_qgemm_split_k_workspace_bytes(int64_t M, int64_t N, int64_t Kexp, int parts) {
    if (M <= 0 || N <= 0 || Kexp <= 0) return 0;
    return qgemm_split_workspace_bytes(M, N, round_up(Kexp, OCS_KALIGN), parts);
}

int ocs_qgemm_split_k(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M, int64_t N,
                      int64_t Kexp, int bits_x, int bits_w, const float* scale_x, const float* scale_w,
                      int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, int parts, void* workspace,
                      size_t ws_bytes, void* stream) {
    if (!Xq || !Wq || !scale_x || !scale_w || !Y) return OCS_E_NULL;
    int rc = check_gemm_operands(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, acc_out, ldacc);
    if (rc) return rc;
    if (ldy < N) return OCS_E_SHAPE;
    const int64_t Kpad = round_up(Kexp, OCS_KALIGN);
    // the K split walks whole K-steps of both operands, also for a short K
    if (ldx < Kpad || ldw < Kpad) return OCS_E_SHAPE;
    if (ldx % OCS_KALIGN != 0 || ldw % OCS_KALIGN != 0) return OCS_E_ALIGN;
    const size_t need = qgemm_split_workspace_bytes(M, N, Kpad, parts);
    if (need == 0) return OCS_E_SHAPE;          // too many tiles, or parts outside 2 .. min(16, K-steps)
    if (workspace == nullptr || ws_bytes < need) return OCS_E_WORKSPACE;
    if (!aligned(workspace, 256)) return OCS_E_ALIGN;
    hipError_t e = launch_qgemm_split(Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w, acc_out, ldacc, Y, ldy,
                                      static_cast<hipStream_t>(stream), parts, workspace);
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_conv_weights_tap_major(const int8_t* Wq, int64_t N, int C_exp, int g, int64_t ldq,
                               int8_t* Wt, int64_t ldc, void* stream) {
    if (!Wq || !Wt) return OCS_E_NULL;
    if (N <= 0 || C_exp <= 0 || g <= 0 || N > (int64_t)1 << 30) return OCS_E_SHAPE;
    if (ldq < (int64_t)C_exp * g || ldc < C_exp || (int64_t)g * ldc > (int64_t)1 << 30) return OCS_E_SHAPE;
    if (ldc % OCS_CALIGN != 0 || !aligned(Wt, 16)) return OCS_E_ALIGN;
    hipError_t e = launch_tap_major(Wq, ldq, N, C_exp, g, ldc, Wt, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_qconv(const int8_t* Aq, int64_t ldc, int B, int H, int W, int C_exp, int kh, int kw,
              int stride, int pad, const int8_t* Wt, int64_t N, int bits_x, int bits_w,
              const float* scale_x, const float* scale_w, int32_t* acc_out, int64_t ldacc, float* Y,
              int64_t ldy, void* stream) {
    if (!Aq || !Wt || !scale_x || !scale_w || !Y) return OCS_E_NULL;
    int rc = check_conv_operands(Aq, ldc, B, H, W, C_exp, kh, kw, stride, pad, Wt, N, bits_x, bits_w,
                                 acc_out, ldacc);
    if (rc) return rc;
    if (ldy < N) return OCS_E_SHAPE;
    hipError_t e = launch_qconv(Aq, ldc, B, H, W, kh, kw, stride, pad, Wt,
                                round_up((int64_t)kh * kw * ldc, OCS_KALIGN), N,
                                scale_x, scale_w, acc_out, ldacc, Y, ldy,
                                static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

static int check_requant(int N, const float* next_threshold, int next_bits,
                         const int32_t* next_chan_src, int next_splits, const int8_t* Yq,
                         int64_t ldyq, const float* next_scale_out) {
    if (!next_threshold || !Yq) return OCS_E_NULL;
    // the kernels keep a workgroup's share of the copies in a table of 512 entries
    if (next_splits < 0 || next_splits > 512 || (int64_t)N + next_splits > OCS_MAX_EXPANDED_CHANNELS)
        return OCS_E_SPLITS;
    if (next_splits > 0 && !next_chan_src) return OCS_E_NULL;
    if (ldyq < (int64_t)N + next_splits) return OCS_E_SHAPE;
    if (ldyq % OCS_CALIGN != 0 || !aligned(Yq, 16)) return OCS_E_ALIGN;
    if (!bits_ok(next_bits)) return OCS_E_BITS;
    if (next_scale_out == next_threshold) return OCS_E_MODE;   // the kernel reads one while writing the other
    return OCS_OK;
}

static Requant make_requant(int relu, const float* next_threshold, int next_bits,
                            const int32_t* next_chan_src, int next_splits, int8_t* Yq,
                            int64_t ldyq, float* next_scale_out) {
    Requant rq;
    rq.Yq = Yq;
    rq.ldyq = ldyq;
    rq.thr = next_threshold;
    rq.qmax = qmax_of(next_bits);
    rq.relu = relu != 0;
    rq.chan_src = next_chan_src;
    rq.s_next = next_splits;
    rq.scale_out = next_scale_out;
    return rq;
}

int ocs_qgemm_requant(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                      int64_t N, int64_t Kexp, int bits_x, int bits_w, const float* scale_x,
                      const float* scale_w, int relu, const float* next_threshold, int next_bits,
                      const int32_t* next_chan_src, int next_splits, int8_t* Yq, int64_t ldyq,
                      float* next_scale_out, int32_t* acc_out, int64_t ldacc, void* stream) {
    if (!Xq || !Wq || !scale_x || !scale_w) return OCS_E_NULL;
    int rc0 = check_gemm_operands(Xq, ldx, Wq, ldw, M, N, Kexp, bits_x, bits_w, acc_out, ldacc);
    if (rc0) return rc0;
    const int64_t Kpad = round_up(Kexp, OCS_KALIGN);
    int rc = check_requant((int)N, next_threshold, next_bits, next_chan_src, next_splits, Yq, ldyq,
                           next_scale_out);
    if (rc) return rc;
    hipError_t e = launch_qgemm(Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w, acc_out, ldacc, nullptr,
                                N, static_cast<hipStream_t>(stream),
                                make_requant(relu, next_threshold, next_bits, next_chan_src,
                                             next_splits, Yq, ldyq, next_scale_out));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_qconv_requant(const int8_t* Aq, int64_t ldc, int B, int H, int W, int C_exp, int kh, int kw,
                      int stride, int pad, const int8_t* Wt, int64_t N, int bits_x, int bits_w,
                      const float* scale_x, const float* scale_w, int relu,
                      const float* next_threshold, int next_bits, const int32_t* next_chan_src,
                      int next_splits, int8_t* Yq, int64_t ldyq, float* next_scale_out,
                      int32_t* acc_out, int64_t ldacc, void* stream) {
    if (!Aq || !Wt || !scale_x || !scale_w) return OCS_E_NULL;
    int rc0 = check_conv_operands(Aq, ldc, B, H, W, C_exp, kh, kw, stride, pad, Wt, N, bits_x, bits_w,
                                  acc_out, ldacc);
    if (rc0) return rc0;
    int rc = check_requant((int)N, next_threshold, next_bits, next_chan_src, next_splits, Yq, ldyq,
                           next_scale_out);
    if (rc) return rc;
    hipError_t e = launch_qconv(Aq, ldc, B, H, W, kh, kw, stride, pad, Wt,
                                round_up((int64_t)kh * kw * ldc, OCS_KALIGN), N, scale_x, scale_w,
                                acc_out, ldacc, nullptr, N, static_cast<hipStream_t>(stream),
                                make_requant(relu, next_threshold, next_bits, next_chan_src,
                                             next_splits, Yq, ldyq, next_scale_out));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_duplicate_weight_codes(int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int num_splits,
                               const int32_t* chan_src, void* stream) {
    if (!Wq || (num_splits > 0 && !chan_src)) return OCS_E_NULL;
    int rc = check_layer(N, C, g, ldq, num_splits);
    if (rc) return rc;
    rc = check_codes(Wq, ldq, (int64_t)(C + num_splits) * g);
    if (rc) return rc;
    hipError_t e = launch_dup_code_columns(Wq, ldq, N, C, g, num_splits, chan_src,
                                           static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_fold_weights(const int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int num_splits,
                     const int32_t* chan_src, int8_t* Wf, int64_t ldf, int32_t* max_abs_out,
                     void* stream) {
    if (!Wq || !Wf || !max_abs_out || (num_splits > 0 && !chan_src)) return OCS_E_NULL;
    int rc = check_layer(N, C, g, ldf, num_splits);
    if (rc) return rc;
    if (ldq < (int64_t)(C + num_splits) * g) return OCS_E_SHAPE;
    rc = check_codes(Wf, ldf, (int64_t)C * g);
    if (rc) return rc;
    hipError_t e = launch_fold_weights(Wq, ldq, N, C, g, num_splits, chan_src, Wf, ldf, max_abs_out,
                                       static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_time_next(int family, void* start_event, void* stop_event) {
    if (family != kTimeSplitQuantize && family != kTimeGemm && family != kTimeAbsmax) return OCS_E_MODE;
    if (!start_event || !stop_event) return OCS_E_NULL;
    KernelTimer& t = kernel_timer();
    t.start[family] = static_cast<hipEvent_t>(start_event);
    t.stop[family] = static_cast<hipEvent_t>(stop_event);
    return OCS_OK;
}

int ocs_calib_copy(const void* src, void* dst, size_t bytes, int workgroups, void* stream) {
    if (!src || !dst) return OCS_E_NULL;
    if (bytes == 0 || bytes % 16 != 0 || workgroups < 0 || workgroups > 65536) return OCS_E_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 16)) return OCS_E_ALIGN;
    if (bytes / 16 / 256 > 0x7FFFFFFFull) return OCS_E_SHAPE;
    hipError_t e = launch_calib_copy(src, dst, bytes, workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_calib_pack(const void* src, void* dst, size_t bytes, int workgroups, void* stream) {
    if (!src || !dst) return OCS_E_NULL;
    if (bytes == 0 || bytes % 16 != 0 || workgroups < 0 || workgroups > 65536) return OCS_E_SHAPE;
    if (bytes / 16 / 256 > 0x7FFFFFFFull) return OCS_E_SHAPE;
    if (!aligned(src, 16) || !aligned(dst, 4)) return OCS_E_ALIGN;
    hipError_t e = launch_calib_pack(src, dst, bytes, workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_calib_read(const void* src, size_t bytes, int passes, int workgroups, void* sink, void* stream) {
    if (!src || !sink) return OCS_E_NULL;
    if (bytes == 0 || bytes % 16 != 0 || passes < 1 || workgroups < 0 || workgroups > 65536) return OCS_E_SHAPE;
    if (workgroups == 0 && (passes != 1 || bytes / 16 / 256 > 0x7FFFFFFFull)) return OCS_E_SHAPE;
    if (passes > 1 && ((bytes / 16) & (bytes / 16 - 1)) != 0) return OCS_E_SHAPE;   // the stream wraps by masking
    if (!aligned(src, 16) || !aligned(sink, 4)) return OCS_E_ALIGN;
    hipError_t e = launch_calib_read(src, bytes, passes, workgroups, sink, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_calib_fill(void* dst, size_t bytes, int value, int nontemporal, int workgroups, void* stream) {
    if (!dst) return OCS_E_NULL;
    if (bytes == 0 || bytes % 16 != 0 || workgroups < 0 || workgroups > 65536) return OCS_E_SHAPE;
    if (bytes / 16 / 256 > 0x7FFFFFFFull) return OCS_E_SHAPE;
    if (!aligned(dst, 16)) return OCS_E_ALIGN;
    hipError_t e = launch_calib_fill(dst, bytes, value, nontemporal, workgroups, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_calib_mfma(const void* operands, int iters, int workgroups, void* sink, void* stream) {
    if (!operands || !sink) return OCS_E_NULL;
    if (iters < 1 || workgroups < 1 || workgroups > 65536) return OCS_E_SHAPE;
    if (!aligned(operands, 16) || !aligned(sink, 4)) return OCS_E_ALIGN;
    hipError_t e = launch_calib_mfma(operands, iters, workgroups, sink, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return OCS_OK;
}

int ocs_tune(const char* key, int value) {
    if (!key) return OCS_E_NULL;
    Tuning& t = tuning();
    if (!strcmp(key, "act_grid")) t.act_grid = value;
    else if (!strcmp(key, "act_nt")) t.act_nt = value < 0 ? 0 : value;
    else if (!strcmp(key, "act_un")) t.act_un = value;
    else if (!strcmp(key, "act_wide")) t.act_wide = value < 0 ? 0 : value;
    else if (!strcmp(key, "act_map")) t.act_map = value;
    else if (!strcmp(key, "act_tile")) t.act_tile = value;
    else if (!strcmp(key, "act_np")) t.act_np = value;
    else if (!strcmp(key, "gemm_tile")) t.gemm_tile = value;
    else if (!strcmp(key, "fused_variant")) t.fused_variant = value;
    else if (!strcmp(key, "fused_stride")) t.fused_stride = value;
    else if (!strcmp(key, "max_flat")) t.max_flat = value;
    else if (!strcmp(key, "max_grid")) t.max_grid = value;
    else if (!strcmp(key, "max_un")) t.max_un = value;
    else if (!strcmp(key, "max_bt")) t.max_bt = value;
    else if (!strcmp(key, "sel_inline")) t.sel_inline = value;
    else if (!strcmp(key, "act_dep")) t.act_dep = value;
    else return OCS_E_MODE;
    return OCS_OK;
}

}  // extern "C"
