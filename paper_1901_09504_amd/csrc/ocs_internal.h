// Internal declarations shared by the translation units of libocs.so (device side only).
// Nothing in here is part of the ABI; see include/ocs.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace ocs {

constexpr int kThreads = 256;      // every kernel here runs 256-thread workgroups (4 wave64)
constexpr int kMaxExpanded = 8000;  // C + s limit of the single-workgroup greedy selector
constexpr int kFlatMaxGrid = 4096;  // most workgroups (= partial maxima) of the flat max|x| pass

typedef float f32x4 __attribute__((ext_vector_type(4)));
// Four consecutive floats at any float address.  Global memory serves a multi-dword access at
// dword alignment, so rows whose length or base is not a multiple of 16 bytes (the 7x7 stem's
// 147-float rows) take the same 16-byte loads as aligned ones.
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Shape of the two-stage column-maximum reduction over a [rows, cols] fp32 tensor.
// Stage 1 writes partial[row_blocks][cols]; stage 2 folds the row blocks into colmax[cols].
struct ReducePlan {
    int vec;            // 4: float4 loads over cols/4 groups (+ scalar pass on cols%4), 1: scalar
    int tx, ty;         // workgroup shape, tx*ty == kThreads
    int col_strips;     // grid.x of the vector pass
    int row_blocks;     // grid.y == number of partial rows
    int rows_per_block; // rows each workgroup walks
};

ReducePlan plan_reduce(int64_t rows, int64_t cols, bool vec_ok);

// Workspace layout (byte offsets from a 256-byte aligned base).
struct Workspace {
    size_t colmax_off;   // float[round_up(cols, 64)]
    size_t partial_off;  // float[max(row_blocks * (cols + 1), kFlatMaxGrid)]
    size_t total;
};
Workspace plan_workspace(int64_t rows, int64_t cols);

// ---- launchers (each returns the hipError_t of its launches) ---------------------------------

// colmax[c] = max_r |T[r, c]| for c < cols.  Two stages, no atomics, deterministic.
hipError_t launch_colmax(const float* T, int64_t rows, int64_t cols, int64_t ld, float* colmax,
                         float* partial, hipStream_t stream);

// scale_out = {T, T/qmax} with T = clip_ratio * max|T| over the whole tensor: the column pass
// with one value per workgroup, then one small reduction (no per-column result).
hipError_t launch_absmax_threshold(const float* T, int64_t rows, int64_t cols, int64_t ld,
                                   float* partial, float clip_ratio, float qmax, float* scale_out,
                                   hipStream_t stream);

// Greedy channel selection (mode 0) or replay of a given split list (mode 1) on the C
// channel maxima derived from colmax[C*g].  Optionally writes max_out and
// scale_out = {clip*max, clip*max/qmax}.
hipError_t launch_select(const float* colmax, int C, int g, int s, int mode,
                         const int32_t* split_in, int32_t* split_src, int32_t* chan_src,
                         int32_t* chan_depth, float* max_out, float clip_ratio, float qmax,
                         float* scale_out, hipStream_t stream);

// scale_out = {T, T/qmax} with T = clip * max over expanded channels j of
// (max_t colmax[chan_src[j]*g+t]) * 2^-chan_depth[j]  (depth NULL: factor 1; src NULL: identity).
hipError_t launch_threshold(const float* colmax, int C, int g, int s, const int32_t* chan_src,
                            const int32_t* chan_depth, float clip_ratio, float qmax,
                            float* scale_out, hipStream_t stream);

// W2 + W3 in one launch for weights (greedy selection repeated by every workgroup, then Eq. 3 and
// Eq. 1): serves few splits on lists of at most 1024 expanded channels, see `..._fits`.  Writes
// what launch_select and launch_expand_quantize together would.
bool select_expand_quantize_fits(int C, int s, int64_t N, int64_t ldq);
hipError_t launch_select_expand_quantize(const float* W, int64_t ldw, int64_t N, int C, int g, int s,
                                         const float* colmax, int32_t* split_src, int32_t* chan_src,
                                         int32_t* chan_depth, float* max_out, float clip_ratio,
                                         float qmax, float* scale_out, int8_t* Wq, int64_t ldq,
                                         hipStream_t stream);

// Fused gather / halve / quantize / pack: the streaming pass over activations (or weights).
// thr: device float threshold; or, with partials != NULL, the threshold is
// clip_ratio * max(partials[0 .. n_partials)), which every workgroup folds for itself.
// scale_out (may be NULL): receives {T, T/qmax}.
// stepwise: the 2^-depth of a channel is applied as `depth` successive halvings (the weights of
// Eq. 3, halved once per split) instead of as one multiply (Eq. 4 on activations with the depth
// given); the two differ only where a result leaves the normal range.
hipError_t launch_expand_quantize(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                  const int32_t* chan_src, const int32_t* chan_depth,
                                  const float* thr, float qmax, int8_t* Xq, int64_t ldq,
                                  float* scale_out, hipStream_t stream,
                                  const float* partials = nullptr, int n_partials = 0,
                                  float clip_ratio = 1.0f, bool stepwise = false);

// Per-workgroup maxima of |T| (stage 1 of the scalar reduction only): partial[0 .. *entries).
hipError_t launch_fold_max(const float* in, int n, float* out, hipStream_t stream);
hipError_t launch_absmax_partials(const float* T, int64_t rows, int64_t cols, int64_t ld,
                                  float* partial, int* entries, hipStream_t stream);

// fp32 expanded tensor: out[r, j*g+t] = T[r, chan_src[j]*g+t] * (halve ? 2^-chan_depth[j] : 1).
hipError_t launch_expand_f32(const float* T, int64_t ld, int64_t rows, int C, int g, int s,
                             const int32_t* chan_src, const int32_t* chan_depth, int halve,
                             float* out, int64_t ldo, hipStream_t stream);

// Sec. 3.3: histories of the expanded channels from the split list, and the QA-split weights
// (fp32 and / or codes rounded by floor(x + 1/2)); scale = {T, T/qmax} as the selector wrote it.
hipError_t launch_qa_paths(const int32_t* split_src, int C, int s, uint32_t* chan_path,
                           hipStream_t stream);
hipError_t launch_dup_code_columns(int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int s,
                                   const int32_t* chan_src, hipStream_t stream);
hipError_t launch_expand_quantize_qa(const float* W, int64_t ldw, int64_t N, int C, int g, int s,
                                     const int32_t* chan_src, const int32_t* chan_depth,
                                     const uint32_t* chan_path, const float* thr, float* scale_out,
                                     float qmax, float* W_out, int64_t ldo, int8_t* Wq, int64_t ldq,
                                     hipStream_t stream);

// Sec. 4.1: maxabs = {m, m / qmax} with m the largest of the n_partials per-workgroup maxima of
// |x| (launch_absmax_partials), histogram of |x| (n_bins <= 8192 bins on [0, m]), error of every
// candidate threshold, out = {first candidate of least error, m}.
hipError_t launch_mse_clip(const float* x, int64_t ldx, int64_t rows, int64_t cols,
                           const float* partials, int n_partials, float* maxabs, int n_bins,
                           int n_cand, float qmax, unsigned long long* hist, double* mse_out,
                           float* out, hipStream_t stream);

// What the GEMM / convolution epilogue may do instead of writing fp32: hand the output to the
// next layer as codes (Eq. 1 with the next layer's static grid, after an optional ReLU, plus
// the copies of the channels the next layer splits: the activation side of its Eq. 3).
// Yq == NULL: plain fp32 output.
struct Requant {
    int8_t* Yq = nullptr;            // [M, ldyq]; columns N + s_next .. ldyq-1 are written as zeros
    int64_t ldyq = 0;
    const float* thr = nullptr;      // device float: the next layer's threshold
    float qmax = 0.0f;
    int relu = 0;
    const int32_t* chan_src = nullptr;   // [N + s_next] (NULL when s_next == 0)
    int s_next = 0;
    float* scale_out = nullptr;      // device float[2] = {T, T/qmax} (may be NULL)
};

// Weight codes of the expanded layer folded onto the C original channels (sum over a channel's
// copies, saturated to +-127); *max_abs = largest |sum|.
hipError_t launch_fold_weights(const int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int s,
                               const int32_t* chan_src, int8_t* Wf, int64_t ldf, int32_t* max_abs,
                               hipStream_t stream);

// int8 x int8 -> int32 MFMA GEMM over Kpad (multiple of 64) with dequantizing epilogue.
hipError_t launch_qgemm(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                        int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                        int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                        hipStream_t stream, const Requant& rq = Requant{});

// The same GEMM with every 256 x 256 tile's K extent shared by `parts` workgroups; partials:
// qgemm_split_workspace_bytes() bytes of device memory (no initialisation needed).
size_t qgemm_split_workspace_bytes(int64_t M, int64_t N, int64_t Kpad, int parts);
hipError_t launch_qgemm_split(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                              int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                              int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream,
                              int parts, void* partials);

// Split + quantize + GEMM in one launch (static grid thr, copies un-scaled as on the activation side
// of Eq. 3): Y = (codes of the expanded X) x Wq^T scaled by (T/qmax) * scale_w[1], without the code
// tensor ever reaching memory.  ..._fits: the shapes it serves (C*g from 64 to 8192, at most 2048
// appended columns, N <= 256).
bool split_act_qgemm_fits(int64_t M, int C, int g, int s, int64_t N, int64_t ldx);
bool split_act_qgemm_pays(int64_t M, int C, int g, int s, int64_t N, int64_t ldx);
hipError_t launch_split_act_qgemm(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                  const int32_t* chan_src, const float* thr, float qmax, const int8_t* Wq,
                                  int64_t ldw, int64_t N, int64_t Kexp, const float* scale_w, float* scale_x_out,
                                  int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream);

// Convolution with the lowering folded into the GEMM's A-operand loader: Aq [B, H, W, ldc]
// codes of the un-lowered activation, Wt [N + 1, kh*kw*ldc] tap-major weight codes whose last
// row is zeros (launch_tap_major builds it from channel-major codes).
hipError_t launch_qconv(const int8_t* Aq, int64_t ldc, int B, int H, int W, int kh, int kw, int stride,
                        int pad, const int8_t* Wt, int64_t ldw, int64_t N, const float* scale_x,
                        const float* scale_w, int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                        hipStream_t stream, const Requant& rq = Requant{});
hipError_t launch_tap_major(const int8_t* Wq, int64_t ldq, int64_t N, int E, int g, int64_t ldc,
                            int8_t* Wt, hipStream_t stream);

// 16-byte copy of `bytes` (multiple of 16) device bytes: counter calibration only.
hipError_t launch_calib_copy(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t stream);
hipError_t launch_calib_pack(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t stream);
// The other measurement kernels (csrc/calib.hip): read-only sweep (passes over the same buffer),
// fill, bare matrix-core loop.
hipError_t launch_calib_read(const void* src, size_t bytes, int passes, int workgroups, void* sink,
                             hipStream_t stream);
hipError_t launch_calib_fill(void* dst, size_t bytes, int value, int nontemporal, int workgroups,
                             hipStream_t stream);
hipError_t launch_calib_mfma(const void* operands, int iters, int workgroups, void* sink, hipStream_t stream);

// A pair of caller-owned events armed for the next launch of one kernel family on this thread:
// that launch goes through hipExtLaunchKernel, which stamps the events with the dispatch's own
// begin and end (what a profiler reports), not with the time of markers around it.
constexpr int kTimeSplitQuantize = 1;
constexpr int kTimeGemm = 2;
constexpr int kTimeAbsmax = 3;
constexpr int kTimeFamilies = 4;
struct KernelTimer {
    hipEvent_t start[kTimeFamilies] = {}, stop[kTimeFamilies] = {};   // one pending pair per family
};
KernelTimer& kernel_timer();

template <typename F, typename... Args>
inline hipError_t launch_kernel(int family, F kernel, dim3 grid, dim3 block, unsigned lds,
                                hipStream_t stream, Args... args) {
    KernelTimer& t = kernel_timer();
    if (family > 0 && family < kTimeFamilies && t.start[family] != nullptr) {
        hipEvent_t a = t.start[family], b = t.stop[family];
        t.start[family] = t.stop[family] = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, a, b, 0, args...);
    } else {
        kernel<<<grid, block, lds, stream>>>(args...);
    }
    return hipGetLastError();
}

// Maximum of a 32-bit unsigned value over the 64 lanes of a wave, returned wave-uniform.  Four
// DPP exchanges fold each row of 16 lanes (pairs, quads, half rows, row); the four row results
// are then read through scalar registers.  Non-negative floats order like their bit patterns.
__device__ __forceinline__ unsigned wave_umax32(unsigned v) {
    unsigned o;
    o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    v = o > v ? o : v;
    o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    v = o > v ? o : v;
    o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    v = o > v ? o : v;
    o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xF, 0xF, false);  // row_mirror
    v = o > v ? o : v;
    const unsigned r0 = (unsigned)__builtin_amdgcn_readlane((int)v, 0);
    const unsigned r1 = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = (unsigned)__builtin_amdgcn_readlane((int)v, 32);
    const unsigned r3 = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    const unsigned a = r0 > r1 ? r0 : r1, b = r2 > r3 ? r2 : r3;
    return a > b ? a : b;
}

// ---- Eq. 1 on the device: shared by the streaming pass and by the GEMM that quantizes its own A operand ----

// One value onto the grid: one fp32 multiply by qmax/T, saturate, round half to even.
// Saturating before rounding gives the same code as rounding first because qmax is an
// integer.  Adding 1.5 * 2^23 rounds |p| <= 127 to an integer under the default rounding mode
// (the sum's ulp is 1) and leaves that integer, in two's complement, in the low mantissa
// bits: the low byte of the sum's bit pattern is the int8 code.
__device__ __forceinline__ unsigned code_bits(float v, float inv_step, float qmax) {
    float p = v * inv_step;
    p = __builtin_amdgcn_fmed3f(p, -qmax, qmax);
    return __float_as_uint(p + 12582912.0f);
}

// low bytes of four words -> one dword (a in byte 0)
__device__ __forceinline__ unsigned pack4(unsigned a, unsigned b, unsigned c, unsigned d) {
    unsigned lo = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);  // {a.b0, b.b0, 0, 0}
    unsigned hi = __builtin_amdgcn_perm(d, c, 0x04000c0cu);  // {0, 0, c.b0, d.b0}
    return lo | hi;
}

// qmax / T as one correctly rounded division, kept finite so that 0 * inv_step stays 0.
__device__ __forceinline__ float inv_step_of(float T, float qmax) {
    if (!(T > 0.0f)) return 0.0f;
    return __builtin_fminf(__fdiv_rn(qmax, T), 3.402823466e+38f);
}

// Launch-shape overrides (benchmarking only); < 0 means "use the default".
struct Tuning {
    int act_grid = -1;  // workgroups of the split+quantize pass
    int act_map = -1;   // lanes of that pass dealt over the output (0), over the input (1), by row shape (-1)
    int act_un = -1;    // items in flight per lane in that pass (1, 2 or 4)
    int act_wide = 0;   // force the 64-bit index variant of that pass (tests: tensors of 2^32 dwords do not fit a test)
    int act_dep = -1;   // Eq. 4 pass: per-column depths from a table in LDS (1), from global memory (0), by tensor size (-1)
    int act_nt = 0;     // non-temporal loads of X in that pass (off: appended columns re-read X through L2)
    int act_np = -1;    // static grid, un-scaled copies: the loop-free flat pass with this many pieces per XCD run (> 0), never (0), by shape (-1)
    int act_tile = -1;  // static grid, un-scaled copies: tile-ordered pass always (1), never (0), by shape (-1)
    int gemm_tile = -1;
    int fused_stride = -1;   // rows between the one-launch kernel's workgroups: forced (> 0), a whole tile always (0), by shape (-1)
    int fused_variant = -1;  // workgroup shape / pipeline depth of the split+quantize+GEMM launch (default: by shape)
    int max_flat = -1;  // whole-tensor max|x| of a contiguous tensor as one flat stream (1), by columns (0), default (-1)
    int max_grid = -1;  // workgroups of the flat pass
    int max_un = -1;    // 16-byte loads in flight per lane in the flat pass (1, 2 or 4)
    int max_bt = -1;    // threads per workgroup of the flat pass (256 or 1024)
    int sel_inline = -1; // most splits for which the weight pass runs the selection itself (0: never; default 16)
};
Tuning& tuning();

}  // namespace ocs
