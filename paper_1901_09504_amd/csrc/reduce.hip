// Column-wise absolute maxima of an fp32 [rows, cols] tensor, and the threshold kernel.
//
// Sec. 3.4 needs, for every input channel, the largest magnitude it holds; Eq. 1 needs the
// largest magnitude of a whole tensor.  Both come from colmax[c] = max_r |T[r,c]|.  The pass
// is bound by HBM: every element is read once with 16-byte loads; the reduction runs in
// registers along rows, through LDS across the rows of a workgroup, and through a small
// partial[row_blocks][cols] buffer across workgroups (no atomics: deterministic, and no
// cross-XCD read-modify-write traffic).
#include "ocs_internal.h"

namespace ocs {

ReducePlan plan_reduce(int64_t rows, int64_t cols, bool vec_ok) {
    ReducePlan p;
    p.vec = (vec_ok && cols >= 4) ? 4 : 1;
    int64_t units = cols / p.vec;
    p.tx = units <= 16 ? 16 : (units <= 32 ? 32 : 64);
    if (p.vec == 4 && units > 32) p.tx = 32;  // 32 lanes x 16 B = 512 B of one row per pass
    p.ty = kThreads / p.tx;
    p.col_strips = (int)ceil_div(units, p.tx);
    // enough workgroups to fill 256 CUs several times over, but a partial buffer of at
    // most ~1 MB so that stage 2 stays negligible
    int64_t want_blocks = ceil_div(2048, p.col_strips);
    int64_t cap_blocks = (int64_t)262144 / (cols > 0 ? cols : 1);
    if (cap_blocks < 16) cap_blocks = 16;
    int64_t rb = want_blocks < cap_blocks ? want_blocks : cap_blocks;
    int64_t max_rb = ceil_div(rows, p.ty);
    if (rb > max_rb) rb = max_rb;
    if (rb < 1) rb = 1;
    // A layer's weights (few rows, long rows): narrow strips that each run down ALL rows give
    // enough workgroups by themselves, and with a single row block stage 1 writes the column
    // maxima directly: one launch instead of two launch-latency-bound ones.
    if (p.vec == 4 && rows <= 2048 && ceil_div(units, 8) >= 32) {
        p.tx = 8;                                  // 8 lanes x 16 B = one 128-byte line per row
        p.ty = kThreads / p.tx;
        p.col_strips = (int)ceil_div(units, p.tx);
        rb = 1;
    }
    p.rows_per_block = (int)ceil_div(rows, rb);
    p.row_blocks = (int)ceil_div(rows, p.rows_per_block);
    return p;
}

Workspace plan_workspace(int64_t rows, int64_t cols) {
    Workspace w;
    // the plan with the most row blocks bounds both the vector and the scalar variant
    ReducePlan a = plan_reduce(rows, cols, true);
    ReducePlan b = plan_reduce(rows, cols, false);
    int64_t rb = a.row_blocks > b.row_blocks ? a.row_blocks : b.row_blocks;
    w.colmax_off = 0;
    w.partial_off = (size_t)round_up(round_up(cols, 64) * 4, 256);
    int64_t entries = rb * (cols + 1);
    if (entries < kFlatMaxGrid) entries = kFlatMaxGrid;
    w.total = w.partial_off + (size_t)round_up(entries * 4, 256);
    return w;
}

// Stage 1.  Workgroup (tx, ty): lane tx owns VEC consecutive columns of strip blockIdx.x,
// ty walks the rows of row block blockIdx.y with stride TY.
// With SCALAR the workgroup folds its columns as well and writes one value,
// partial[blockIdx.y * gridDim.x + blockIdx.x]: enough when only the tensor's maximum is wanted.
template <int VEC, bool SCALAR>
__global__ __launch_bounds__(kThreads) void colmax_partial_kernel(
    const float* __restrict__ T, int64_t ld, int64_t rows, int64_t col0, int64_t units,
    int rows_per_block, int64_t out_cols, float* __restrict__ partial) {
    __shared__ float red[kThreads * VEC];
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const int64_t u = (int64_t)blockIdx.x * TX + tx;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > rows) r1 = rows;

    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;

    if (u < units) {
        const float* base = T + col0 + u * VEC;
#pragma unroll 4
        for (int64_t r = r0 + ty; r < r1; r += TY) {
            if constexpr (VEC == 4) {
                // a plain load, not a non-temporal one: the pass that follows (split+quantize)
                // reads the same tensor again, and lines loaded with the streaming hint are not
                // kept in the 256 MB memory-side cache (measured: this pass 1.5 us slower, the
                // next one 4 us faster on a 115 MB tensor)
                f32x4 v = *reinterpret_cast<const f32x4u*>(base + r * ld);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = fmaxf(acc[e], fabsf(v[e]));
            } else {
                acc[0] = fmaxf(acc[0], fabsf(base[r * ld]));
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[(ty * TX + tx) * VEC + e] = acc[e];
    __syncthreads();
    if (SCALAR) {
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) m = fmaxf(m, acc[e]);
        const int t = ty * TX + tx;
        __syncthreads();
        red[t] = m;
        __syncthreads();
        for (int w = kThreads / 2; w > 0; w >>= 1) {
            if (t < w) red[t] = fmaxf(red[t], red[t + w]);
            __syncthreads();
        }
        if (t == 0) partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = red[0];
        return;
    }
    if (ty == 0 && u < units) {
        for (int y = 1; y < TY; ++y)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = fmaxf(acc[e], red[(y * TX + tx) * VEC + e]);
        float* dst = partial + (int64_t)blockIdx.y * out_cols + col0 + u * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[e] = acc[e];
    }
}

// max|x| of a contiguous tensor as ONE flat stream: lane i of the grid reads 16-byte groups
// i, i + G, i + 2G, ..., UN of them in flight, so that at any moment the chip reads one
// compact window that slides over the tensor.  A read-only stream is fastest with about 8 MB
// in flight (measured on 0.4 to 1.8 GB buffers: 6.1 TB/s; with four times as much in flight
// 5.2-5.5 TB/s), which the row-block layout of the column pass above does not give.  One
// value per workgroup, partial[blockIdx.x], and few workgroups (one of 1024 lanes per CU): the
// pass that follows folds the partial maxima once per workgroup of its own, and 2000 of them
// cost it 1.3 us more than 256 do.
template <int UN, int BT>
__global__ __launch_bounds__(BT) void absmax_flat_kernel(const float* __restrict__ x, int64_t n,
                                                         float* __restrict__ partial) {
    __shared__ float red[BT / 64];
    const f32x4u* x4 = reinterpret_cast<const f32x4u*>(x);
    const int64_t n4 = n / 4;
    const int64_t stride = (int64_t)gridDim.x * BT;
    float m = 0.0f;
    int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x;
    for (; i + (UN - 1) * stride < n4; i += UN * stride) {
        f32x4 v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) v[u] = x4[i + u * stride];
#pragma unroll
        for (int u = 0; u < UN; ++u)
            m = fmaxf(fmaxf(fmaxf(m, fabsf(v[u][0])), fmaxf(fabsf(v[u][1]), fabsf(v[u][2]))), fabsf(v[u][3]));
    }
    for (; i < n4; i += stride) {
        const f32x4 v = x4[i];
        m = fmaxf(fmaxf(fmaxf(m, fabsf(v[0])), fmaxf(fabsf(v[1]), fabsf(v[2]))), fabsf(v[3]));
    }
    // the n % 4 last elements
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(n - 4 * n4)) m = fmaxf(m, fabsf(x[4 * n4 + threadIdx.x]));
    const unsigned w = wave_umax32(__float_as_uint(m));   // magnitudes: non-negative, order like unsigned
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = __uint_as_float(w);
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = red[0];
#pragma unroll
        for (int k = 1; k < BT / 64; ++k) r = fmaxf(r, red[k]);
        partial[blockIdx.x] = r;
    }
}

// out[0] = max of the n non-negative floats at in.  One workgroup: for a pass that would otherwise
// fold the maxima once per workgroup of its own and has a great many small workgroups.
constexpr int kFoldThreads = 1024;
__global__ __launch_bounds__(kFoldThreads) void fold_max_kernel(const float* __restrict__ in, int n,
                                                                float* __restrict__ out) {
    __shared__ float red[kFoldThreads / 64];
    float m = 0.0f;
    for (int i = threadIdx.x; i < n; i += kFoldThreads) m = fmaxf(m, in[i]);
    const unsigned w = wave_umax32(__float_as_uint(m));   // magnitudes: non-negative, order like unsigned
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = __uint_as_float(w);
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = red[0];
#pragma unroll
        for (int k = 1; k < kFoldThreads / 64; ++k) r = fmaxf(r, red[k]);
        out[0] = r;
    }
}

hipError_t launch_fold_max(const float* in, int n, float* out, hipStream_t stream) {
    fold_max_kernel<<<1, kFoldThreads, 0, stream>>>(in, n, out);
    return hipGetLastError();
}

// Stage 2: colmax[c] = max over partial rows.  Workgroup = 64 columns x 4 row groups.
__global__ __launch_bounds__(kThreads) void colmax_final_kernel(const float* __restrict__ partial,
                                                                int row_blocks, int64_t cols,
                                                                float* __restrict__ colmax) {
    __shared__ float red[kThreads];
    const int cx = threadIdx.x & 63, gy = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + cx;
    float m = 0.0f;
    if (c < cols) {
#pragma unroll 8
        for (int r = gy; r < row_blocks; r += 4) m = fmaxf(m, partial[(int64_t)r * cols + c]);
    }
    red[threadIdx.x] = m;
    __syncthreads();
    if (gy == 0 && c < cols) {
        m = fmaxf(fmaxf(red[cx], red[64 + cx]), fmaxf(red[128 + cx], red[192 + cx]));
        colmax[c] = m;
    }
}

static hipError_t launch_partials(const float* T, int64_t rows, int64_t cols, int64_t ld,
                                  float* partial, bool scalar, const ReducePlan& p, int* entries,
                                  hipStream_t stream) {
    dim3 block(p.tx, p.ty);
    int n = 0;
    if (p.vec == 4) {
        int64_t units = cols / 4;
        dim3 grid(p.col_strips, p.row_blocks);
        if (scalar) {
            hipError_t te = launch_kernel(kTimeAbsmax, colmax_partial_kernel<4, true>, grid, block, 0,
                                          stream, T, ld, rows, (int64_t)0, units, p.rows_per_block,
                                          cols, partial);
            if (te != hipSuccess) return te;
        } else
            colmax_partial_kernel<4, false><<<grid, block, 0, stream>>>(T, ld, rows, 0, units,
                                                                        p.rows_per_block, cols, partial);
        n = p.col_strips * p.row_blocks;
        int64_t left = cols - units * 4;
        if (left > 0) {  // the last cols % 4 columns, one lane each
            dim3 grid1(1, p.row_blocks);
            if (scalar)
                colmax_partial_kernel<1, true><<<grid1, block, 0, stream>>>(
                    T, ld, rows, units * 4, left, p.rows_per_block, cols, partial + n);
            else
                colmax_partial_kernel<1, false><<<grid1, block, 0, stream>>>(
                    T, ld, rows, units * 4, left, p.rows_per_block, cols, partial);
            n += p.row_blocks;
        }
    } else {
        dim3 grid(p.col_strips, p.row_blocks);
        if (scalar)
            colmax_partial_kernel<1, true><<<grid, block, 0, stream>>>(T, ld, rows, 0, cols,
                                                                       p.rows_per_block, cols, partial);
        else
            colmax_partial_kernel<1, false><<<grid, block, 0, stream>>>(T, ld, rows, 0, cols,
                                                                        p.rows_per_block, cols, partial);
        n = p.col_strips * p.row_blocks;
    }
    if (entries) *entries = n;
    return hipGetLastError();
}

hipError_t launch_colmax(const float* T, int64_t rows, int64_t cols, int64_t ld, float* colmax,
                         float* partial, hipStream_t stream) {
    const bool vec_ok = true;   // 16-byte loads at the float's own alignment (f32x4u)
    ReducePlan p = plan_reduce(rows, cols, vec_ok);
    if (p.row_blocks == 1)   // a single row block: stage 1's output is the result
        return launch_partials(T, rows, cols, ld, colmax, false, p, nullptr, stream);
    hipError_t e = launch_partials(T, rows, cols, ld, partial, false, p, nullptr, stream);
    if (e != hipSuccess) return e;
    colmax_final_kernel<<<(unsigned)ceil_div(cols, 64), kThreads, 0, stream>>>(partial, p.row_blocks,
                                                                              cols, colmax);
    return hipGetLastError();
}

// scale_out = {T, T/qmax}, T = clip_ratio * max(v[0..n)).  One workgroup.
__global__ __launch_bounds__(kThreads) void threshold_scalar_kernel(const float* __restrict__ v, int n,
                                                                    float clip_ratio, float qmax,
                                                                    float* __restrict__ scale_out) {
    __shared__ float red[kThreads];
    float m = 0.0f;
    for (int i = threadIdx.x; i < n; i += kThreads) m = fmaxf(m, v[i]);
    red[threadIdx.x] = m;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float T = clip_ratio * red[0];
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
}

// The flat pass when the tensor is one contiguous range (ld == cols); *entries = workgroups.
static bool launch_absmax_flat(const float* T, int64_t rows, int64_t cols, int64_t ld, float* partial,
                               int* entries, hipStream_t stream, hipError_t* err) {
    const int want = tuning().max_flat;
    if (ld != cols || want == 0) return false;
    const int64_t n = rows * cols;
    const int bt = tuning().max_bt == 256 ? 256 : 1024;
    int64_t grid = tuning().max_grid > 0 ? tuning().max_grid : 256;
    if (grid > kFlatMaxGrid) grid = kFlatMaxGrid;
    if (grid > ceil_div(ceil_div(n, 4), bt)) grid = ceil_div(ceil_div(n, 4), bt);
    if (grid < 1) grid = 1;
    const int un = tuning().max_un < 0 ? 2 : tuning().max_un;
    const dim3 g((unsigned)grid), b(bt);
#define OCS_FLAT(U, T_) *err = launch_kernel(kTimeAbsmax, absmax_flat_kernel<U, T_>, g, b, 0, stream, T, n, partial)
    if (bt == 256) {
        if (un == 4) OCS_FLAT(4, 256); else if (un == 2) OCS_FLAT(2, 256); else OCS_FLAT(1, 256);
    } else {
        if (un == 4) OCS_FLAT(4, 1024); else if (un == 2) OCS_FLAT(2, 1024); else OCS_FLAT(1, 1024);
    }
#undef OCS_FLAT
    if (entries) *entries = (int)grid;
    return true;
}

hipError_t launch_absmax_partials(const float* T, int64_t rows, int64_t cols, int64_t ld,
                                  float* partial, int* entries, hipStream_t stream) {
    hipError_t fe = hipSuccess;
    if (launch_absmax_flat(T, rows, cols, ld, partial, entries, stream, &fe)) return fe;
    const bool vec_ok = true;   // 16-byte loads at the float's own alignment (f32x4u)
    ReducePlan p = plan_reduce(rows, cols, vec_ok);
    return launch_partials(T, rows, cols, ld, partial, true, p, entries, stream);
}

hipError_t launch_absmax_threshold(const float* T, int64_t rows, int64_t cols, int64_t ld,
                                   float* partial, float clip_ratio, float qmax, float* scale_out,
                                   hipStream_t stream) {
    const bool vec_ok = true;   // 16-byte loads at the float's own alignment (f32x4u)
    ReducePlan p = plan_reduce(rows, cols, vec_ok);
    int n = 0;
    hipError_t e = hipSuccess;
    if (!launch_absmax_flat(T, rows, cols, ld, partial, &n, stream, &e))
        e = launch_partials(T, rows, cols, ld, partial, true, p, &n, stream);
    if (e != hipSuccess) return e;
    threshold_scalar_kernel<<<1, kThreads, 0, stream>>>(partial, n, clip_ratio, qmax, scale_out);
    return hipGetLastError();
}

// Threshold of Eq. 1 for an expanded activation tensor without materialising it:
// max_j (channel maximum of chan_src[j]) * 2^-chan_depth[j], times the clip ratio.
__global__ __launch_bounds__(kThreads) void threshold_kernel(
    const float* __restrict__ colmax, int C, int g, int s, const int32_t* __restrict__ chan_src,
    const int32_t* __restrict__ chan_depth, float clip_ratio, float qmax,
    float* __restrict__ scale_out) {
    __shared__ float red[kThreads];
    float m = 0.0f;
    if (chan_depth == nullptr) {
        // copies do not change the maximum: plain maximum over all columns
        for (int64_t c = threadIdx.x; c < (int64_t)C * g; c += kThreads) m = fmaxf(m, colmax[c]);
    } else {
        for (int j = threadIdx.x; j < C + s; j += kThreads) {
            int src = chan_src ? chan_src[j] : j;
            src = src < 0 ? 0 : (src >= C ? C - 1 : src);
            float cm = 0.0f;
            for (int t = 0; t < g; ++t) cm = fmaxf(cm, colmax[(int64_t)src * g + t]);
            m = fmaxf(m, cm * ldexpf(1.0f, -chan_depth[j]));
        }
    }
    red[threadIdx.x] = m;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        float T = clip_ratio * red[0];
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
}

hipError_t launch_threshold(const float* colmax, int C, int g, int s, const int32_t* chan_src,
                            const int32_t* chan_depth, float clip_ratio, float qmax,
                            float* scale_out, hipStream_t stream) {
    threshold_kernel<<<1, kThreads, 0, stream>>>(colmax, C, g, s, chan_src, chan_depth, clip_ratio,
                                                 qmax, scale_out);
    return hipGetLastError();
}

}  // namespace ocs
