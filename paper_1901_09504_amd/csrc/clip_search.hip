// Clip threshold of least mean squared error (Sec. 4.1), a calibration-time routine.
//
// A histogram h of |x| over n equal bins on [0, m], m = max|x|; a bin counts at its centre
// x_i; for each of n_cand thresholds T_c = m * c / n_cand the error
// MSE(T_c) = 1/n * sum_i h_i * (x_i - Q_{T_c}(x_i))^2 with the quantizer of Eq. 1; the first
// candidate with the least error is the result.  Bin decisions and codes are taken in fp32
// with the same operation order as everywhere else in the library; errors are accumulated in
// fp64 over the bins in increasing order, one candidate per lane, so that the choice does not
// depend on how the work is spread over workgroups.
#include "ocs_internal.h"

namespace ocs {

// Set-up in one launch: the histogram cleared, and {m, m / qmax} from the per-workgroup maxima
// that the max|x| pass left behind (first workgroup).
__global__ __launch_bounds__(kThreads) void mse_prepare_kernel(const float* __restrict__ partials, int n,
                                                               float qmax, float* __restrict__ maxabs_out,
                                                               unsigned long long* __restrict__ hist,
                                                               int n_bins) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n_bins) hist[i] = 0ull;
    if (blockIdx.x != 0) return;
    __shared__ unsigned red[kThreads / 64];
    float m = 0.0f;
    for (int k = threadIdx.x; k < n; k += kThreads) m = fmaxf(m, partials[k]);
    const unsigned w = wave_umax32(__float_as_uint(m));      // maxima of magnitudes: non-negative
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned u = red[0];
#pragma unroll
        for (int q = 1; q < kThreads / 64; ++q) u = red[q] > u ? red[q] : u;
        const float T = __uint_as_float(u);
        maxabs_out[0] = T;
        maxabs_out[1] = T / qmax;
    }
}

// Frequencies: each workgroup counts in LDS, then adds its counts to the global histogram
// (integer sums: any order gives the same result).  Few, large workgroups (one of 1024 lanes per
// CU): every workgroup ends with one global atomic per non-empty bin, and with a thousand small
// workgroups those two million atomics on two thousand addresses were most of the pass.
constexpr int kHistThreads = 1024;
__global__ __launch_bounds__(kHistThreads) void hist_kernel(const float* __restrict__ x, int64_t ldx,
                                                            int64_t rows, int64_t cols,
                                                            const float* __restrict__ maxabs, int n_bins,
                                                            unsigned long long* __restrict__ hist) {
    extern __shared__ unsigned int lhist[];
    for (int i = threadIdx.x; i < n_bins; i += kHistThreads) lhist[i] = 0u;
    __syncthreads();
    const float m = maxabs[0];
    float to_bin = 0.0f;
    if (m > 0.0f) to_bin = __builtin_fminf(__fdiv_rn((float)n_bins, m), 3.402823466e+38f);
    const int64_t total = rows * cols;
    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    const bool flat16 = ldx == cols && total % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
    if (flat16) {       // one contiguous, 16-byte aligned range: four values per load
        const f32x4* x4 = reinterpret_cast<const f32x4*>(x);
        // the next 16 bytes are requested before this item's four counts go to LDS
        const int64_t n4 = total / 4;
        int64_t e = (int64_t)blockIdx.x * kHistThreads + threadIdx.x;
        f32x4 v = x4[e < n4 ? e : 0];
        for (; e < n4; e += stride) {
            const f32x4 nxt = x4[e + stride < n4 ? e + stride : e];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float p = fabsf(v[k]) * to_bin;
                const int b = p >= (float)n_bins ? n_bins - 1 : (int)p;
                atomicAdd(&lhist[b], 1u);
            }
            v = nxt;
        }
    } else {
        for (int64_t e = (int64_t)blockIdx.x * kHistThreads + threadIdx.x; e < total; e += stride) {
            const int64_t r = e / cols, c = e - r * cols;
            const float p = fabsf(x[r * ldx + c]) * to_bin;
            const int b = p >= (float)n_bins ? n_bins - 1 : (int)p;
            atomicAdd(&lhist[b], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < n_bins; i += kHistThreads)
        if (lhist[i] != 0u) atomicAdd(&hist[i], (unsigned long long)lhist[i]);
}

// Error of every candidate: 64 candidates per workgroup, one per lane.  A candidate's sum runs
// over the bins in increasing order (that order is part of the result), but the terms of the sum
// are independent: fifteen of the workgroup's sixteen waves each work out the terms of two bins
// of a chunk of 30 for all 64 candidates and leave them in LDS, while the first wave adds the
// previous chunk's 30 terms to its running sums in bin order (two sets of terms, used
// alternately, one barrier per chunk).  (With one wave doing both for all bins the sweep was bound
// by that single wave's instruction issue: 2048 bins x 512 candidates took ~85 us on eight busy
// waves in the whole chip; with terms and sums taking turns, 37 us.)
constexpr int kSweepWaves = 16, kSweepBinsPerWave = 2;
constexpr int kSweepChunk = (kSweepWaves - 1) * kSweepBinsPerWave;

template <bool STAGED>
__global__ __launch_bounds__(kSweepWaves * 64) void mse_sweep_kernel(
    const unsigned long long* __restrict__ hist, const float* __restrict__ maxabs, int n_bins,
    int n_cand, float qmax, double* __restrict__ mse_out) {
    __shared__ double term[2][kSweepChunk][64];
    // the frequencies as doubles in LDS, fetched once (a load per chunk on the spot, with its
    // wait, cost more than the arithmetic); left in global memory only when they do not fit
    extern __shared__ double hd[];
    if (STAGED) {
        for (int i = threadIdx.x; i < n_bins; i += kSweepWaves * 64) hd[i] = (double)hist[i];
        __syncthreads();
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane + 1;     // lanes past n_cand compute and store nothing useful
    const float m = maxabs[0];
    const float width = __fdiv_rn(m, (float)n_bins);
    const float T = m * __fdiv_rn((float)c, (float)n_cand);
    float inv = 0.0f;
    if (T > 0.0f) inv = __builtin_fminf(__fdiv_rn(qmax, T), 3.402823466e+38f);
    const float step = __fdiv_rn(T, qmax);
    // waves 1..15: this wave's two terms of the chunk that starts at bin `base`
    auto produce = [&](int base, int buf) {
#pragma unroll
        for (int k = 0; k < kSweepBinsPerWave; ++k) {
            const int b = (wave - 1) * kSweepBinsPerWave + k, i = base + b;
            double t = 0.0;
            if (i < n_bins) {
                const float xi = ((float)i + 0.5f) * width;
                float code = rintf(xi * inv);
                code = code > qmax ? qmax : code;
                code = code < -qmax ? -qmax : code;
                const double e = (double)xi - (double)code * (double)step;
                t = (STAGED ? hd[i] : (double)hist[i]) * (e * e);
            }
            term[buf][b][lane] = t;
        }
    };
    if (wave > 0) produce(0, 0);
    __syncthreads();
    double sum = 0.0;
    int buf = 0;
    for (int base = 0; base < n_bins; base += kSweepChunk) {
        if (wave == 0) {
            double t[kSweepChunk];
#pragma unroll
            for (int b = 0; b < kSweepChunk; ++b) t[b] = term[buf][b][lane];
            // the additions stay in bin order; bins past the last one contribute +0.0, which
            // leaves a sum of non-negative terms as it is
#pragma unroll
            for (int b = 0; b < kSweepChunk; ++b) sum += t[b];
        } else if (base + kSweepChunk < n_bins) {
            produce(base + kSweepChunk, buf ^ 1);
        }
        __syncthreads();
        buf ^= 1;
    }
    if (wave == 0 && c <= n_cand) mse_out[c - 1] = __ddiv_rn(sum, (double)n_bins);
}

// The first candidate of least error.  One workgroup; lane t looks at candidates t+1,
// t+1+256, ... in increasing order; the lanes' bests then meet in a tree in LDS whose every
// node keeps the smaller error and, among equal errors, the earlier candidate.
__global__ __launch_bounds__(kThreads) void mse_argmin_kernel(const double* __restrict__ mse,
                                                              const float* __restrict__ maxabs,
                                                              int n_cand, float* __restrict__ out) {
    __shared__ double best_err[kThreads];
    __shared__ int best_c[kThreads];
    double my_err = 0.0;
    int my_c = 0;          // 0: this lane has seen no candidate
    for (int c = threadIdx.x + 1; c <= n_cand; c += kThreads) {
        const double err = mse[c - 1];
        if (my_c == 0 || err < my_err) {
            my_err = err;
            my_c = c;
        }
    }
    best_err[threadIdx.x] = my_err;
    best_c[threadIdx.x] = my_c;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            const int ca = best_c[threadIdx.x], cb = best_c[threadIdx.x + w];
            const double ea = best_err[threadIdx.x], eb = best_err[threadIdx.x + w];
            const bool take_b = cb != 0 && (ca == 0 || eb < ea || (eb == ea && cb < ca));
            if (take_b) {
                best_err[threadIdx.x] = eb;
                best_c[threadIdx.x] = cb;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float m = maxabs[0];
        out[0] = m * __fdiv_rn((float)best_c[0], (float)n_cand);
        out[1] = m;
    }
}

hipError_t launch_mse_clip(const float* x, int64_t ldx, int64_t rows, int64_t cols,
                           const float* partials, int n_partials, float* maxabs, int n_bins,
                           int n_cand, float qmax, unsigned long long* hist, double* mse_out,
                           float* out, hipStream_t stream) {
    mse_prepare_kernel<<<dim3((unsigned)ceil_div(n_bins, kThreads)), kThreads, 0, stream>>>(
        partials, n_partials, qmax, maxabs, hist, n_bins);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int64_t grid = ceil_div(rows * cols, (int64_t)kHistThreads * 16);
    if (grid > 256) grid = 256;
    if (grid < 1) grid = 1;
    hist_kernel<<<dim3((unsigned)grid), kHistThreads, (size_t)n_bins * sizeof(unsigned int), stream>>>(
        x, ldx, rows, cols, maxabs, n_bins, hist);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // the staged frequencies and the 30 KB of terms share the 64 KB a workgroup gets without
    // opting in to more
    const size_t staged_bytes = (size_t)n_bins * sizeof(double);
    if (staged_bytes + sizeof(double) * 2 * kSweepChunk * 64 + 256 <= 65536)
        mse_sweep_kernel<true><<<dim3((unsigned)ceil_div(n_cand, 64)), kSweepWaves * 64, staged_bytes, stream>>>(
            hist, maxabs, n_bins, n_cand, qmax, mse_out);
    else
        mse_sweep_kernel<false><<<dim3((unsigned)ceil_div(n_cand, 64)), kSweepWaves * 64, 0, stream>>>(
            hist, maxabs, n_bins, n_cand, qmax, mse_out);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    mse_argmin_kernel<<<1, kThreads, 0, stream>>>(mse_out, maxabs, n_cand, out);
    return hipGetLastError();
}

}  // namespace ocs
