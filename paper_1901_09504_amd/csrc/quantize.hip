// The fused split + quantize pass (Sec. 3.5's "copy and scale the chosen channels" layer
// followed by Eq. 1), and the fp32 materialisation of an expanded tensor.
//
// One streaming pass, bound by HBM: 4 bytes read and (1+r) bytes written per element.
// Each lane turns 16 bytes of fp32 input into one packed dword of four int8 codes.  The first
// C*g output columns of a row are an identity gather (16-byte loads); only the s*g appended
// columns gather from elsewhere in the same row, which the workgroup has just pulled through
// the caches, so no element of X is fetched from HBM twice.  With Eq. 3 (weights carry the
// halving) the appended codes are byte copies of their source codes; with Eq. 4 every
// expanded channel j is scaled by 2^-chan_depth[j] before it meets the grid.
#include <atomic>

#include "ocs_internal.h"
#include "select_lds.h"

namespace ocs {

// v halved d times, one halving after the other, as the splits of Sec. 3.4 are performed on the
// weights (Eq. 3 per split).  While the result stays a normal number that is one exact multiply
// by 2^-d; a result below the normal range rounds at every further halving, which a single
// multiply would not reproduce.
__device__ __forceinline__ float halved(float v, int d) {
    const int e = (int)((__float_as_uint(v) >> 23) & 0xFFu);      // biased exponent
    if (d <= 126 && e > d) return v * ldexpf(1.0f, -d);           // exponent e - d >= 1: exact
    if (d <= 0) return v;
    int h = e - 1;                                                // halvings that keep it normal
    h = h < 0 ? 0 : (h > d ? d : h);
    float r = v;
    if (h > 0) {
        const int h1 = h < 126 ? h : 126;
        r = r * ldexpf(1.0f, -h1);
        if (h > h1) r = r * ldexpf(1.0f, -(h - h1));
    }
    for (int i = h; i < d && r != 0.0f; ++i) r = r * 0.5f;       // at most ~25 roundings before zero
    return r;
}

// The threshold of the pass: the given device float, or, for a per-batch grid, clip_ratio times
// the largest of the per-workgroup maxima the preceding pass left behind (a few thousand
// floats, folded by every workgroup for itself: cheaper than a separate launch that does only
// that).  All lanes return the same value; contains a barrier.
__device__ __forceinline__ float pass_threshold(const float* thr, const float* partials, int n,
                                                float clip_ratio, float* red /* >= 4 floats of LDS */) {
    if (partials == nullptr) {
        const float T = *thr;
        __syncthreads();
        return T;
    }
    float m = 0.0f;
    for (int i = threadIdx.x; i < n; i += kThreads) m = fmaxf(m, partials[i]);
    const unsigned w = wave_umax32(__float_as_uint(m));      // maxima of magnitudes: non-negative
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = __uint_as_float(w);
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    return clip_ratio * m;
}

// Eq. 4's per-channel factors for the contiguous region of a row, as one byte per column in LDS:
// dep_col[k] = halvings of the channel that column k belongs to (255 stands for any larger count:
// 2^-150 and below already round to zero as an fp32 factor).  Built once per workgroup, channel by
// channel, so that the pass needs no division by g and no look-up in global memory per element.
__device__ __forceinline__ void build_depth_table(unsigned char* dep_col, const int32_t* __restrict__ chan_depth,
                                                  int C, int g) {
    for (int j = threadIdx.x; j < C; j += kThreads) {
        const int dj = chan_depth[j];
        const unsigned char b = (unsigned char)(dj < 0 ? 0 : (dj > 255 ? 255 : dj));
        for (int t = 0; t < g; ++t) dep_col[j * g + t] = b;
    }
}
// v[e] * 2^-dep of columns 4d .. 4d+3 (a multiply by an exact power of two, as ldexpf(1, -dep) gives it)
__device__ __forceinline__ void scale_by_depth(f32x4& v, const unsigned char* dep_col, int d) {
    const unsigned dd = *reinterpret_cast<const unsigned*>(dep_col + 4 * d);
    if (dd != 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] * ldexpf(1.0f, -(int)((dd >> (8 * e)) & 0xFFu));
    }
}

template <bool NT>
__device__ __forceinline__ f32x4 load4(const f32x4u* p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

// One lane per packed output dword, the whole output walked as ONE flat range with a grid
// stride: lane i of the grid produces dwords i, i + G, i + 2G, ...  Consecutive lanes read
// consecutive 16-byte groups of X and write consecutive dwords of Xq, and at any moment the
// whole chip works inside one compact window that slides over X front to back, which is the
// access pattern HBM serves fastest (measured against row-per-wave and row-per-workgroup
// layouts with LDS staging of the appended columns; those were 10-15 % slower).
//   d <  main_units: the dword's four inputs are the contiguous X[r, 4d .. 4d+3], one 16-byte
//                    load at whatever alignment the row has (main_units = K / 4);
//   d >= main_units: leftover columns, appended channels (their source values were fetched
//                    moments ago by neighbouring lanes, so the re-read is served by the
//                    caches, not by HBM) and the zero padding.
constexpr int kTailTable = 2048;  // appended + padded columns whose sources are kept in LDS
constexpr int kDepthTableMax = 16384;  // widest unexpanded row whose per-column depths are kept in LDS (1 B each)

template <bool HALVE, bool NT, int UN, typename Index>
__global__ __launch_bounds__(kThreads) void expand_quantize_kernel(
    const float* __restrict__ X, int64_t ldx, int64_t M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth,
    const float* thr, float qmax, int8_t* __restrict__ Xq, int D, int main_units,
    unsigned magic, float* scale_out, const float* __restrict__ partials, int n_partials,
    float clip_ratio, int dep_table, int stepwise) {
    // stepwise (weights, Eq. 3 applied split by split): 2^-depth as `halved` applies it; otherwise
    // (activations, Eq. 4 with the depth given) one multiply by 2^-depth.  dep_table is then 0.
    __shared__ float thr_red[kThreads / 64];
    // Source column (or -1 for padding) and halving depth of every column past the vector
    // region.  They do not depend on the row, so each workgroup resolves them once; a lane that
    // lands on such a column then needs a single trip to memory, like every other lane.
    __shared__ __align__(16) int tail_col[kTailTable];
    __shared__ int tail_dep[HALVE ? kTailTable : 1];
    extern __shared__ __align__(16) unsigned char dep_col[];   // HALVE and dep_table: one byte per column
    if (HALVE && dep_table) build_depth_table(dep_col, chan_depth, C, g);
    const int Ke = (C + s) * g;
    const int tail0 = 4 * main_units;              // first column of the gather region
    const int tail_n = 4 * D - tail0;              // columns in it (appended, leftover, padding)
    const bool use_table = tail_n <= kTailTable;
    if (use_table) {
        for (int e = threadIdx.x; e < tail_n; e += kThreads) {
            const int k = tail0 + e;
            int col = -1, dep = 0;
            if (k < Ke) {
                const int j = k / g, t = k - j * g;
                int src = chan_src ? chan_src[j] : j;
                src = src < 0 ? 0 : (src >= C ? C - 1 : src);
                col = src * g + t;
                if (HALVE) dep = chan_depth[j];
            }
            tail_col[e] = col;
            if (HALVE) tail_dep[e] = dep;
        }
    }
    const Index total = (Index)M * (Index)D;
    const Index stride = (Index)gridDim.x * kThreads;
    unsigned* __restrict__ out = reinterpret_cast<unsigned*>(Xq);

    // Position of output dword o.  With 32-bit indices the division by D is a multiply by
    // magic = floor(2^32 / D) and one correction step (the estimate is never more than one low).
    auto locate = [&](Index o, Index& row, int& d) {
        if (sizeof(Index) == 4) {
            unsigned q = __umulhi((unsigned)o, magic);
            unsigned r = (unsigned)o - q * (unsigned)D;
            if (r >= (unsigned)D) { ++q; r -= (unsigned)D; }
            row = (Index)q;
            d = (int)r;
        } else {
            row = o / (Index)D;
            d = (int)(o - row * (Index)D);
        }
    };
    // requests the 16-byte input of item o (if it has one) and remembers where the item lives
    auto fetch = [&](Index o, f32x4& v, Index& row, int& d) {
        row = 0;
        d = 0;
        if (o < total) {
            locate(o, row, d);
            if (d < main_units)
                v = load4<NT>(reinterpret_cast<const f32x4u*>(X + (int64_t)row * ldx) + d);
        }
    };

    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber them
    // so that neighbouring 1 KB pieces of a row are read through the same L2: the lanes that
    // gather appended columns then find their source values in that L2 instead of asking
    // HBM for the line a second time.
    const unsigned nwg = gridDim.x, xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const unsigned vwg = xcd * (nwg / 8) + (xcd < nwg % 8 ? xcd : nwg % 8) + slot;

    // One item: quantize, pack and store output dword o (row, d), whose 16-byte input, if it
    // has one, is already in v.
    auto emit = [&](Index o, Index row, int d, const f32x4& vin, float inv) {
        const float* xrow = X + (int64_t)row * ldx;
        unsigned q;
        if (d < main_units) {
            f32x4 v = vin;
            if (HALVE && dep_table) {
                scale_by_depth(v, dep_col, d);
            } else if (HALVE) {
                int j = (4 * d) / g, t = 4 * d - j * g;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = stepwise ? halved(v[e], chan_depth[j]) : v[e] * ldexpf(1.0f, -chan_depth[j]);
                    if (++t == g) { t = 0; ++j; }
                }
            }
            q = pack4(code_bits(v[0], inv, qmax), code_bits(v[1], inv, qmax),
                      code_bits(v[2], inv, qmax), code_bits(v[3], inv, qmax));
        } else {
            float v[4];
            int dep[4];
            const int e0 = 4 * (d - main_units);
            if (use_table) {
                // one 16-byte read of the four source columns; the loads are unconditional
                // (a padding column reads column 0 and discards it): branch-free, so that a wave
                // with a few lanes here does not run four masked branches for all 64
                const i32x4 cols = *reinterpret_cast<const i32x4*>(&tail_col[e0]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int col = cols[e];
                    dep[e] = HALVE ? tail_dep[e0 + e] : 0;
                    const float x = xrow[col < 0 ? 0 : col];
                    v[e] = col >= 0 ? x : 0.0f;
                }
            } else {
                const int k = 4 * d;
                int j = k / g, t = k - j * g;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = 0.0f;
                    dep[e] = 0;
                    if (k + e < Ke) {
                        int src = chan_src ? chan_src[j] : j;
                        src = src < 0 ? 0 : (src >= C ? C - 1 : src);
                        v[e] = xrow[(int64_t)src * g + t];
                        if (HALVE) dep[e] = chan_depth[j];
                    }
                    if (++t == g) { t = 0; ++j; }
                }
            }
            if (HALVE) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = stepwise ? halved(v[e], dep[e]) : v[e] * ldexpf(1.0f, -dep[e]);
            }
            q = pack4(code_bits(v[0], inv, qmax), code_bits(v[1], inv, qmax),
                      code_bits(v[2], inv, qmax), code_bits(v[3], inv, qmax));
        }
        out[o] = q;
    };

    // Each trip of a lane covers UN items, stride apart; the inputs of the next trip are
    // requested before this trip's items are processed.  The first inputs are requested before
    // anything waits on the threshold.
    Index o = (Index)vwg * kThreads + threadIdx.x;
    f32x4 cur[UN] = {}, nxt[UN] = {};
    Index row[UN] = {}, nrow[UN] = {};
    int d[UN] = {}, nd[UN] = {};
#pragma unroll
    for (int u = 0; u < UN; ++u) fetch(o + (Index)u * stride, cur[u], row[u], d[u]);
    const float T = pass_threshold(thr, partials, n_partials, clip_ratio, thr_red);  // + barrier
    const float inv = inv_step_of(T, qmax);
    if (scale_out != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }

    for (; o < total; o += (Index)UN * stride) {
#pragma unroll
        for (int u = 0; u < UN; ++u)
            fetch(o + (Index)(UN + u) * stride, nxt[u], nrow[u], nd[u]);
#pragma unroll
        for (int u = 0; u < UN; ++u)
            if (o + (Index)u * stride < total) emit(o + (Index)u * stride, row[u], d[u], cur[u], inv);
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            cur[u] = nxt[u];
            row[u] = nrow[u];
            d[u] = nd[u];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The pass in one shot, for a static grid with un-scaled copies (the activation side of Eq. 3): a
// workgroup takes R whole rows (a few KB of X), requests all of its input at once (U 16-byte loads
// per lane), turns it into codes, and is done: no loop, no look-ahead registers, one barrier.  The
// chip's dispatcher hands such workgroups out in order, so the chip works inside one tight window
// that slides over X, tighter than persistent workgroups keep it (they drift apart): a plain copy
// written this way moves 6.0 TB/s on this chip against 5.5 TB/s for the grid-stride form, and this
// pass's pattern of 16 bytes in and 4 out per lane 6.1 against 5.5 (the library's measurement
// kernels, calib.hip).
//   Main items: dword d < Qc = ceil(K/4) of a row, 16 bytes of X each; their codes go straight to
//   memory (d < Q = floor(K/4)) and into an image of the rows in LDS.
//   Tail: dwords Q .. D-1 of a row (left-over columns of X, the appended columns, zero padding)
//   are assembled afterwards from the image, byte by byte: the copy of a column is the code just
//   written, so the appended columns cost no second trip to memory.  Their source columns do not
//   depend on the row: a table of 4 * TD entries, looked up in chan_src behind the requests for X.
// ---------------------------------------------------------------------------------------------
constexpr int kShotNT = 256;
constexpr int kShotTabPer = 2;                       // table entries per lane
constexpr int kShotMaxTail = kShotNT * kShotTabPer;  // tail columns 4 * TD served

template <int U>
__global__ __launch_bounds__(kShotNT) void expand_quantize_shot_kernel(
    const float* __restrict__ X, int64_t ldx, int M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const float* __restrict__ thr, float qmax,
    int8_t* __restrict__ Xq, int64_t ldq, int R, unsigned magic_qc, unsigned magic_td,
    float* __restrict__ scale_out, float clip) {
    // clip: the threshold is clip * *thr (1 for a given threshold; the clip ratio when *thr is the
    // tensor's largest magnitude, left behind by the pass before this one)
    extern __shared__ __align__(16) int8_t slds[];
    const int K = C * g, Q = K / 4, rem = K - 4 * Q, Qc = Q + (rem > 0 ? 1 : 0);
    const int D = (int)(ldq / 4), TD = D - Q, Ke = (C + s) * g;
    const int P = (int)ldq + 4;                       // image pitch: consecutive rows start one bank apart
    int8_t* img = slds;
    int* tcol = reinterpret_cast<int*>(slds + ((R * P + 15) & ~15));
    const int tid = (int)threadIdx.x;
    const int row0 = (int)blockIdx.x * R;
    const int rows = M - row0 < R ? M - row0 : R;

    // the table's look-ups first: they come back from the L2 while the rows are on their way
    int tsrc[kShotTabPer];
#pragma unroll
    for (int i = 0; i < kShotTabPer; ++i) {
        const int k = 4 * Q + tid + i * kShotNT;
        const bool app = k >= K && k < Ke;
        tsrc[i] = chan_src != nullptr ? chan_src[app ? k / g : 0] : 0;     // (no list: no appended columns)
    }
    // main items: item i = (row i / Qc, dword i % Qc)
    f32x4 v[U];
    int r_[U], d_[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = tid + u * kShotNT;
        unsigned q = __umulhi((unsigned)i, magic_qc);           // floor(i / Qc), at most one low
        unsigned d = (unsigned)i - q * (unsigned)Qc;
        if (d >= (unsigned)Qc) { ++q; d -= (unsigned)Qc; }
        const bool ok = (int)q < rows;
        r_[u] = ok ? (int)q : -1;
        d_[u] = (int)d;
        // a row's last dword may hold fewer than four columns of X: it is fetched as the row's last
        // four floats and shifted into place when used (nothing is read past the row)
        const float* src = X + (int64_t)(row0 + (ok ? (int)q : 0)) * ldx + (ok ? ((int)d < Q ? 4 * (int)d : K - 4) : 0);
        v[u] = *reinterpret_cast<const f32x4u*>(src);
    }
#pragma unroll
    for (int i = 0; i < kShotTabPer; ++i) {
        const int e = tid + i * kShotNT, k = 4 * Q + e;
        if (e < 4 * TD) {
            int col = -1;
            if (k < K) col = k;
            else if (k < Ke) {
                const int j = k / g, t = k - j * g;
                const int c = tsrc[i] < 0 ? 0 : (tsrc[i] >= C ? C - 1 : tsrc[i]);
                col = c * g + t;
            }
            tcol[e] = col;
        }
    }
    const float T = clip * *thr;
    const float inv = inv_step_of(T, qmax);
    if (scale_out != nullptr && blockIdx.x == 0 && tid == 0) {
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
    unsigned* __restrict__ out = reinterpret_cast<unsigned*>(Xq);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (r_[u] < 0) continue;
        unsigned q4 = pack4(code_bits(v[u][0], inv, qmax), code_bits(v[u][1], inv, qmax),
                            code_bits(v[u][2], inv, qmax), code_bits(v[u][3], inv, qmax));
        if (d_[u] < Q) out[(int64_t)(row0 + r_[u]) * D + d_[u]] = q4;
        else q4 >>= 8 * (4 - rem);                     // columns 4Q .. K-1 are the fetched elements 4-rem .. 3
        *reinterpret_cast<unsigned*>(img + r_[u] * P + 4 * d_[u]) = q4;
    }
    __syncthreads();
    for (int it = tid; it < rows * TD; it += kShotNT) {
        unsigned r = __umulhi((unsigned)it, magic_td);          // floor(it / TD), at most one low
        unsigned td = (unsigned)it - r * (unsigned)TD;
        if (td >= (unsigned)TD) { ++r; td -= (unsigned)TD; }
        const i32x4 cols = *reinterpret_cast<const i32x4*>(&tcol[4 * td]);
        const int8_t* irow = img + (int)r * P;
        unsigned q4 = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned byte = (unsigned)(unsigned char)irow[cols[e] < 0 ? 0 : cols[e]];
            q4 |= (cols[e] < 0 ? 0u : byte) << (8 * e);
        }
        out[(int64_t)(row0 + (int)r) * D + Q + (int)td] = q4;
    }
}

struct ShotPlan {
    int U = 0, R = 0;
};
// Rows per workgroup and loads per lane.  Measured on the paper's layer shapes at batch 256: a
// workgroup is fastest with about 512 main items (two loads per lane, 8 KB of X); rows too long
// for two of them to fit take three loads' worth (e.g. two rows of 288 items), and a single long
// row whatever it needs, up to 8 loads per lane.  force_u > 0: that many loads per lane, with as
// many rows as they hold (tests and tuning).
constexpr int kShotMaxU = 8;
static ShotPlan shot_plan(int64_t M, int64_t K, int64_t ldq, int force_u = 0) {
    ShotPlan p;
    if (M < 1 || M > 0x7FFFFFFF - 4096 || K < 4 || K > 4 * kShotNT * kShotMaxU || ldq % 16 != 0) return p;
    const int64_t Q = K / 4, Qc = (K + 3) / 4, TD = ldq / 4 - Q;
    if (TD < 0 || 4 * TD > kShotMaxTail) return p;
    int64_t R;
    if (force_u > 0) {
        R = (int64_t)kShotNT * force_u / Qc;
        if (R < 1) return p;
    } else {
        R = 512 / Qc;
        if (R * Qc < 448) R = 768 / Qc;
        if (R < 1) R = 1;
    }
    if (R > 64) R = 64;
    p.R = (int)R;
    p.U = force_u > 0 ? force_u : (int)ceil_div(R * Qc, kShotNT);
    if (p.U > kShotMaxU) p = ShotPlan{};
    return p;
}

template <int U>
static hipError_t run_expand_quantize_shot(const ShotPlan& p, const float* X, int64_t ldx, int64_t M, int C, int g,
                                           int s, const int32_t* chan_src, const float* thr, float qmax, int8_t* Xq,
                                           int64_t ldq, float* scale_out, hipStream_t stream, float clip) {
    const int64_t K = (int64_t)C * g, Q = K / 4, Qc = (K + 3) / 4, TD = ldq / 4 - Q;
    // floor(2^32 / n), or 2^32 - 1 for n = 1: the quotient estimate is then at most one low, which
    // the kernel's correction step absorbs
    auto magic_of = [](int64_t n) {
        const uint64_t m = (((uint64_t)1) << 32) / (uint64_t)n;
        return (unsigned)(m > 0xFFFFFFFFull ? 0xFFFFFFFFull : m);
    };
    const unsigned magic_qc = magic_of(Qc);
    const unsigned magic_td = TD > 0 ? magic_of(TD) : 0u;
    const unsigned lds = (unsigned)(((p.R * (ldq + 4) + 15) & ~(int64_t)15) + (TD > 0 ? 4 * TD : 1) * 4);
    return launch_kernel(kTimeSplitQuantize, expand_quantize_shot_kernel<U>, dim3((unsigned)ceil_div(M, p.R)),
                         dim3(kShotNT), lds, stream, X, ldx, (int)M, C, g, s, chan_src, thr, qmax, Xq, ldq, p.R,
                         magic_qc, magic_td, scale_out, clip);
}

// The same pass with the lanes dealt over the INPUT instead: one lane per 16-byte group of X,
// the whole of X walked as one flat range, so every lane of every load instruction carries
// data (in the output-ordered kernel above the lanes that land on appended columns and on the
// padding load nothing, which for narrow rows is half of them).  Lane (row, d) writes output
// dword d of its row and, when d < TD = D - Q, also dword Q + d: an appended or padding dword,
// whose sources it gathers from the same row (the K % 4 leftover columns are among them).
// Q = K/4 groups per row; requires 1 <= TD <= Q.
template <bool HALVE, typename Index>
__global__ __launch_bounds__(kThreads) void expand_quantize_in_kernel(
    const float* __restrict__ X, int64_t ldx, int64_t M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth,
    const float* thr, float qmax, int8_t* __restrict__ Xq, int D, int Q, unsigned magic,
    float* scale_out, const float* __restrict__ partials, int n_partials, float clip_ratio,
    int dep_table) {
    __shared__ float thr_red[kThreads / 64];
    __shared__ __align__(16) int tail_col[kTailTable];
    __shared__ int tail_dep[HALVE ? kTailTable : 1];
    extern __shared__ __align__(16) unsigned char dep_col[];   // HALVE and dep_table: one byte per column
    if (HALVE && dep_table) build_depth_table(dep_col, chan_depth, C, g);
    const int Ke = (C + s) * g;
    const int TD = D - Q;                          // appended + padding dwords per row
    for (int e = threadIdx.x; e < 4 * TD; e += kThreads) {
        const int k = 4 * Q + e;
        int col = -1, dep = 0;
        if (k < Ke) {
            const int j = k / g, t = k - j * g;
            int src = chan_src ? chan_src[j] : j;
            src = src < 0 ? 0 : (src >= C ? C - 1 : src);
            col = src * g + t;
            if (HALVE) dep = chan_depth[j];
        }
        tail_col[e] = col;
        if (HALVE) tail_dep[e] = dep;
    }
    const Index total = (Index)M * (Index)Q;
    const Index stride = (Index)gridDim.x * kThreads;
    unsigned* __restrict__ out = reinterpret_cast<unsigned*>(Xq);

    auto locate = [&](Index o, Index& row, int& d) {
        if (sizeof(Index) == 4) {
            unsigned q = __umulhi((unsigned)o, magic);
            unsigned r = (unsigned)o - q * (unsigned)Q;
            if (r >= (unsigned)Q) { ++q; r -= (unsigned)Q; }
            row = (Index)q;
            d = (int)r;
        } else {
            row = o / (Index)Q;
            d = (int)(o - row * (Index)Q);
        }
    };
    auto fetch_main = [&](Index o, f32x4& v, Index& row, int& d) {
        row = 0;
        d = 0;
        if (o < total) {
            locate(o, row, d);
            v = *(reinterpret_cast<const f32x4u*>(X + (int64_t)row * ldx) + d);
        }
    };
    auto fetch_tail = [&](Index o, Index row, int d, f32x4& tv) {
        if (o < total && d < TD) {
            const float* xrow = X + (int64_t)row * ldx;
            const i32x4 cols = *reinterpret_cast<const i32x4*>(&tail_col[4 * d]);
            // a dword of padding alone (all four columns -1) requests nothing: with narrow rows most
            // tail dwords are that, and their lanes would all ask for their row's first element
            if ((cols[0] & cols[1] & cols[2] & cols[3]) >= 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {     // unconditional loads: see the output-ordered kernel
                    const int col = cols[e];
                    const float x = xrow[col < 0 ? 0 : col];
                    tv[e] = col >= 0 ? x : 0.0f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) tv[e] = 0.0f;
            }
        }
    };

    const unsigned nwg = gridDim.x, xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const unsigned vwg = xcd * (nwg / 8) + (xcd < nwg % 8 ? xcd : nwg % 8) + slot;

    auto emit = [&](Index row, int d, f32x4 v, f32x4 tv, float inv) {
        const Index base = row * (Index)D;
        if (HALVE && dep_table) {
            scale_by_depth(v, dep_col, d);
        } else if (HALVE) {
            int j = (4 * d) / g, t = 4 * d - j * g;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = v[e] * ldexpf(1.0f, -chan_depth[j]);
                if (++t == g) { t = 0; ++j; }
            }
        }
        out[base + (Index)d] = pack4(code_bits(v[0], inv, qmax), code_bits(v[1], inv, qmax),
                                     code_bits(v[2], inv, qmax), code_bits(v[3], inv, qmax));
        if (d < TD) {
            if (HALVE) {
#pragma unroll
                for (int e = 0; e < 4; ++e) tv[e] = tv[e] * ldexpf(1.0f, -tail_dep[4 * d + e]);
            }
            out[base + (Index)(Q + d)] =
                pack4(code_bits(tv[0], inv, qmax), code_bits(tv[1], inv, qmax),
                      code_bits(tv[2], inv, qmax), code_bits(tv[3], inv, qmax));
        }
    };

    Index o = (Index)vwg * kThreads + threadIdx.x;
    f32x4 cur = {}, nxt = {}, tcur = {}, tnxt = {};
    Index row = 0, nrow = 0;
    int d = 0, nd = 0;
    fetch_main(o, cur, row, d);       // requested before anything waits on the threshold
    const float T = pass_threshold(thr, partials, n_partials, clip_ratio, thr_red);
    const float inv = inv_step_of(T, qmax);
    if (scale_out != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
    // (the barrier inside pass_threshold also completes the column table)
    fetch_tail(o, row, d, tcur);

    for (; o < total; o += stride) {
        fetch_main(o + stride, nxt, nrow, nd);
        fetch_tail(o + stride, nrow, nd, tnxt);
        emit(row, d, cur, tcur, inv);
        cur = nxt;
        tcur = tnxt;
        row = nrow;
        d = nd;
    }
}

// ---------------------------------------------------------------------------------------------
// The pass in tile order, for a static grid with un-scaled copies (the activation side of Eq. 3):
// a workgroup of 4 waves takes 64 rows and builds their expanded code rows in LDS, then writes
// them out as one contiguous block (the rows of Xq follow each other at the pitch).  It walks the
// columns of X in steps of 64: every lane requests four 16-byte pieces one step ahead (each load
// instruction of a wave covers four rows' whole 256 bytes) and turns the previous step's 16
// floats into codes at their place in the image.  The appended columns never touch memory on the
// way: the copy of a column is the byte that has just been written into LDS, so after each step
// the copies whose sources it holds are moved inside the image, byte by byte.
// ---------------------------------------------------------------------------------------------
__device__ __align__(16) int8_t tile_zero_chunk[16] = {};   // what a lane with nothing to fetch reads

struct TileLds {
    int pitch, first_off, cursor_off, ent_off, total;
};
constexpr int kTileNT = 256;
constexpr int kTileMaxTail = 2048;
constexpr int kTileMaxLds = 72 * 1024;     // two workgroups per compute unit

static TileLds tile_lds(int BM, int64_t ldq, int ksteps_main, int T) {
    TileLds l;
    // image rows hold the pitch rounded up to whole steps, plus 16 bytes so that consecutive rows
    // start in different banks
    l.pitch = (int)round_up(ldq, 64) + 16;
    l.first_off = BM * l.pitch;
    l.cursor_off = l.first_off + (ksteps_main + 2) * 4;
    l.ent_off = l.cursor_off + (ksteps_main + 1) * 4;
    l.total = l.ent_off + (T > 0 ? T : 1) * 4;
    return l;
}

template <int BM, int WPE, int SETS>
__global__ __launch_bounds__(kTileNT, WPE) void expand_quantize_tile_kernel(
    const float* __restrict__ X, int64_t ldx, int M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const float* __restrict__ thr, float qmax,
    int8_t* __restrict__ Xq, int64_t ldq, int ksteps_main, int rem, float* __restrict__ scale_out, TileLds L) {
    // ksteps_main: whole 64-column steps of X; rem: columns of X left over after them (< 64)
    constexpr int NT = kTileNT, A_PER = BM * 16 / NT;
    static_assert(A_PER >= 1 && A_PER * NT == BM * 16, "the threads tile a step of X");
    extern __shared__ __align__(1024) int8_t tlds[];
    int8_t* img = tlds;                                          // [BM][pitch]: code of expanded column j at [r][j]
    int* first = reinterpret_cast<int*>(tlds + L.first_off);     // [ksteps_main + 2]
    int* cursor = reinterpret_cast<int*>(tlds + L.cursor_off);   // [ksteps_main + 1]
    int* ent = reinterpret_cast<int*>(tlds + L.ent_off);         // [T]: (e << 6) | source column inside its step
    const int P = L.pitch;

    const int tid = (int)threadIdx.x;
    const int row0 = (int)blockIdx.x * BM;
    const int T = s * g, K = ksteps_main * 64 + rem;

    // the step's BM x 16 float4 numbered row-major; load i of thread t is number i*NT + t
    const float* a_src[A_PER];
    int a_dst[A_PER];
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int f = i * NT + tid, r = f >> 4, f4 = f & 15;
        int gr = row0 + r;
        gr = gr < M ? gr : M - 1;          // rows past the edge re-read the last row; never stored
        a_src[i] = X + (int64_t)gr * ldx + f4 * 4;
        a_dst[i] = r * P + f4 * 4;
    }
    f32x4 av[SETS][A_PER];   // SETS register sets in rotation: SETS-1 steps are on their way while one is processed
    auto load_step = [&](int kt, f32x4 (&a)[A_PER]) {
        // every lane issues the same loads at every step (a lane with nothing to fetch reads the 16
        // zero bytes): no branch around a load, so the look-ahead stays in flight across the waits
        const bool main_step = kt < ksteps_main, rest_step = kt == ksteps_main && rem > 0;
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int c0 = ((i * NT + tid) & 15) * 4;
            // left-over columns: a float4 that would cross the row's end starts four floats before
            // the end instead and is shifted into place when it is used
            const bool whole = main_step || (rest_step && c0 + 3 < rem);
            const bool part = rest_step && c0 < rem && !whole;
            const float* src = whole ? a_src[i] + (int64_t)kt * 64
                                     : (part ? a_src[i] + (int64_t)kt * 64 - c0 + (rem - 4)
                                             : reinterpret_cast<const float*>(tile_zero_chunk));
            a[i] = *reinterpret_cast<const f32x4u*>(src);
        }
    };
#pragma unroll
    for (int p = 0; p + 1 < SETS; ++p) load_step(p, av[p]);

    {   // behind the first requests: zero the rows' ends (columns past X's own: what no copy fills is
        // padding), bucket the appended columns by the step of their source
        const int z0 = ksteps_main * 64, zn = (P - 16 - z0) / 4;           // dwords per row from column z0 on
        for (int o = tid; o < BM * zn; o += NT) {
            const int r = o / zn, c = o - r * zn;
            *reinterpret_cast<int*>(img + r * P + z0 + 4 * c) = 0;
        }
        for (int k = tid; k <= ksteps_main + 1; k += NT) first[k] = 0;
        __syncthreads();
        for (int e = tid; e < T; e += NT) {
            const int j = e / g, t = e - j * g;
            int src = chan_src[C + j];
            src = src < 0 ? 0 : (src >= C ? C - 1 : src);
            atomicAdd(&first[((src * g + t) >> 6) + 1], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int run = 0;
            for (int k = 0; k <= ksteps_main; ++k) {
                run += first[k + 1];
                first[k + 1] = run;
            }
        }
        __syncthreads();
        for (int k = tid; k <= ksteps_main; k += NT) cursor[k] = first[k];
        __syncthreads();
        for (int e = tid; e < T; e += NT) {
            const int j = e / g, t = e - j * g;
            int src = chan_src[C + j];
            src = src < 0 ? 0 : (src >= C ? C - 1 : src);
            const int col = src * g + t;
            const int pos = atomicAdd(&cursor[col >> 6], 1);
            ent[pos] = (e << 6) | (col & 63);
        }
        // (the first step's barrier completes the table before anyone reads it)
    }
    const float Tx = *thr;
    const float inv = inv_step_of(Tx, qmax);
    if (scale_out != nullptr && blockIdx.x == 0 && tid == 0) {
        scale_out[0] = Tx;
        scale_out[1] = Tx / qmax;
    }

    auto process = [&](int kt, const f32x4 (&a)[A_PER]) {
        const bool main_step = kt < ksteps_main;
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const unsigned q4 = pack4(code_bits(a[i][0], inv, qmax), code_bits(a[i][1], inv, qmax),
                                      code_bits(a[i][2], inv, qmax), code_bits(a[i][3], inv, qmax));
            int8_t* dst = img + a_dst[i] + kt * 64;
            const int c0 = ((i * NT + tid) & 15) * 4;
            if (main_step || c0 + 3 < rem) {
                *reinterpret_cast<unsigned*>(dst) = q4;
            } else {
                // left-over columns at the row's end: byte by byte (the dword also holds copies).  The
                // float4 was fetched as columns rem-4 .. rem-1 of the step: this lane's column
                // c0 + e is its element c0 + e - (rem - 4)
                const int d = c0 - (rem - 4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c0 + e < rem) dst[e] = (int8_t)((q4 >> (8 * (e + d))) & 0xFFu);
            }
        }
        __syncthreads();
        // the copies whose sources this step holds: one byte per (copy, row), to expanded column K + e
        const int e0 = first[kt], n = first[kt + 1] - e0;
        for (int idx = tid; idx < n * BM; idx += NT) {
            const int q = idx / BM, r = idx - q * BM;
            const int en = ent[e0 + q];
            img[r * P + K + (en >> 6)] = img[r * P + kt * 64 + (en & 63)];
        }
    };

    const int steps = ksteps_main + (rem > 0 ? 1 : 0);
    for (int kt0 = 0; kt0 < steps; kt0 += SETS) {
#pragma unroll
        for (int p = 0; p < SETS; ++p) {
            const int kt = kt0 + p;
            if (kt < steps) {
                load_step(kt + SETS - 1, av[(p + SETS - 1) % SETS]);
                process(kt, av[p]);
            }
        }
    }
    __syncthreads();   // the image is complete
    // out as one contiguous block: 16-byte piece o of the block is piece o % (ldq/16) of row o / (ldq/16)
    const int ppr = (int)(ldq / 16);
    const int rows = M - row0 < BM ? M - row0 : BM;
    i32x4* out = reinterpret_cast<i32x4*>(Xq + (int64_t)row0 * ldq);
    for (int o = tid; o < rows * ppr; o += NT) {
        const int r = o / ppr, c = o - r * ppr;
        out[o] = *reinterpret_cast<const i32x4*>(img + r * P + c * 16);
    }
}

// Shapes the tile-ordered pass serves: the image of 64 expanded rows has to leave room for two
// workgroups per compute unit.
static bool tile_fits(int64_t M, int64_t K, int64_t T, int64_t ldq) {
    if (M < 1 || M > 0x7FFFFFFF - 64 || K < 64 || T > kTileMaxTail || ldq % 16 != 0 || ldq > 65536) return false;
    return tile_lds(64, ldq, (int)(K / 64), (int)T).total <= kTileMaxLds;
}

template <int BM, int SETS>
static hipError_t run_expand_quantize_tile(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                           const int32_t* chan_src, const float* thr, float qmax, int8_t* Xq,
                                           int64_t ldq, float* scale_out, hipStream_t stream) {
    const int64_t K = (int64_t)C * g;
    const int ksteps_main = (int)(K / 64), rem = (int)(K - (int64_t)ksteps_main * 64);
    const TileLds L = tile_lds(BM, ldq, ksteps_main, s * g);
    static std::atomic<bool> opted_in[64];
    if (L.total > 65536) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (!opted_in[dev].load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&expand_quantize_tile_kernel<BM, 4, SETS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kTileMaxLds);
            if (e != hipSuccess) return e;
            opted_in[dev].store(true, std::memory_order_release);
        }
    }
    return launch_kernel(kTimeSplitQuantize, expand_quantize_tile_kernel<BM, 4, SETS>, dim3((unsigned)ceil_div(M, BM)),
                         dim3(kTileNT), (unsigned)L.total, stream, X, ldx, (int)M, C, g, s, chan_src, thr, qmax, Xq, ldq,
                         ksteps_main, rem, scale_out, L);
}

hipError_t launch_expand_quantize(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                  const int32_t* chan_src, const int32_t* chan_depth,
                                  const float* thr, float qmax, int8_t* Xq, int64_t ldq,
                                  float* scale_out, hipStream_t stream, const float* partials,
                                  int n_partials, float clip_ratio, bool stepwise) {
    const int64_t K = (int64_t)C * g;
    const bool vec_ok = true;   // 16-byte loads need only the float's own alignment
    const int main_units = (int)(K / 4);
    const int D = (int)(ldq / 4);
    const int64_t total = M * D;
    const bool nt = tuning().act_nt != 0;
    const bool halve = chan_depth != nullptr;
    // Eq. 4: the per-column depth table in LDS, one byte per column of the unexpanded row, when a
    // lane has enough items for the table's set-up to pay (weights, with one or two items per lane,
    // were 0.6-2.3 us slower with it; cfg 2's activations, with 14, are 5 us faster)
    const bool dep_pays = tuning().act_dep < 0 ? M * (ldq / 4) >= (int64_t)8 * 2048 * kThreads : tuning().act_dep != 0;
    const int dep_table = halve && !stepwise && K <= kDepthTableMax && dep_pays ? 1 : 0;
    const unsigned dep_lds = dep_table ? (unsigned)round_up(K, 16) : 0;

    int64_t grid = 256 * 8;  // 8 workgroups of 4 waves on each of the 256 CUs
    if (tuning().act_grid > 0) grid = tuning().act_grid;
    if (grid > ceil_div(total, kThreads)) grid = ceil_div(total, kThreads);
    // Static grid, un-scaled copies: the one-shot pass wherever it serves the shape (measured against
    // the tile-ordered and the flat passes below on the paper's layer shapes at batch 256: 1-13 % ahead
    // on every one of them)
    // (except rows of fewer than 256 values that are not whole 16-byte groups, the 7x7 stem's 147: a
    // third of such a workgroup's items are tail dwords, and the tile-ordered pass below, which writes
    // its image out in 16-byte pieces, is 6 % ahead there)
    const int np_mode = tuning().act_np;
    const bool odd_narrow = K % 4 != 0 && K < 256 && tile_fits(M, K, (int64_t)s * g, ldq);
    // (a per-batch grid whose pass before this one left the maximum itself behind, one entry, is served
    // too: the threshold is then the clip ratio times that entry)
    const bool given = thr != nullptr && partials == nullptr, one_max = thr == nullptr && partials != nullptr && n_partials == 1;
    if ((given || one_max) && !halve && (chan_src != nullptr || s == 0) && np_mode != 0 && tuning().act_tile <= 0 &&
        tuning().act_map < 0 && (np_mode > 0 || !odd_narrow)) {
        const ShotPlan p = shot_plan(M, K, ldq, np_mode > 0 && np_mode <= kShotMaxU ? np_mode : 0);
#define OCS_SHOT_ARGS p, X, ldx, M, C, g, s, chan_src, given ? thr : partials, qmax, Xq, ldq, scale_out, stream, given ? 1.0f : clip_ratio
        switch (p.U) {
            case 1: return run_expand_quantize_shot<1>(OCS_SHOT_ARGS);
            case 2: return run_expand_quantize_shot<2>(OCS_SHOT_ARGS);
            case 3: return run_expand_quantize_shot<3>(OCS_SHOT_ARGS);
            case 4: return run_expand_quantize_shot<4>(OCS_SHOT_ARGS);
            case 5: return run_expand_quantize_shot<5>(OCS_SHOT_ARGS);
            case 6: return run_expand_quantize_shot<6>(OCS_SHOT_ARGS);
            case 7: return run_expand_quantize_shot<7>(OCS_SHOT_ARGS);
            case 8: return run_expand_quantize_shot<8>(OCS_SHOT_ARGS);
            default: break;     // a shape it does not serve: the passes below
        }
#undef OCS_SHOT_ARGS
    }
    // Static grid, un-scaled copies: the tile-ordered pass.  Measured against the flat orders below on
    // the paper's layer shapes at batch 256 (inside the whole pass over the network): 4-17 % ahead for
    // rows of X up to 256 values, and up to 576 on very tall X (the flat pass's gather lanes stall
    // their waves there, and a row's end is written as a few scattered bytes); level or behind for
    // 512-value rows on shorter X, level at 1152, behind from 1024-value 1x1 rows on.
    // Two steps of look-ahead (level with one), one for rows of a single step.
    const int tile_mode = tuning().act_tile;
    if (thr != nullptr && partials == nullptr && !halve && tile_mode != 0 &&
        tile_fits(M, K, (int64_t)s * g, ldq) &&
        (tile_mode > 0 || ldq <= 320 || (ldq <= 768 && M >= 400000))) {
        if (K < 128) return run_expand_quantize_tile<64, 2>(X, ldx, M, C, g, s, chan_src, thr, qmax, Xq, ldq, scale_out, stream);
        return run_expand_quantize_tile<64, 3>(X, ldx, M, C, g, s, chan_src, thr, qmax, Xq, ldq, scale_out, stream);
    }

    // Lanes dealt over the input when its rows allow it (see expand_quantize_in_kernel)
    const int Q = main_units, TD = D - Q;
    // Measured: it wins (up to 1.45x) once a quarter or more of a row's output dwords are
    // appended columns or padding (rows of 64 to 128 values); for wider rows the two are level.
    const int map = tuning().act_map;
    const bool by_input = map < 0 ? (4 * TD >= D || Q <= 16) : map != 0;
    if (by_input && !stepwise && vec_ok && Q >= 1 && TD <= Q && 4 * TD <= kTailTable) {
        const int64_t total_in = M * Q;
        int64_t gin = 256 * 8;
        if (tuning().act_grid > 0) gin = tuning().act_grid;
        if (gin > ceil_div(total_in, kThreads)) gin = ceil_div(total_in, kThreads);
        // output dword indices reach M*D; the prefetch looks two strides past the item
        const bool wide_in = tuning().act_wide > 0 || total + 2 * gin * kThreads >= ((int64_t)1 << 32);
        const unsigned magic_q = (unsigned)((((uint64_t)1) << 32) / (uint64_t)Q);
#define OCS_LAUNCH_IN(H, I_)                                                                       \
    launch_kernel(kTimeSplitQuantize, expand_quantize_in_kernel<H, I_>, dim3((unsigned)gin),      \
                  dim3(kThreads), dep_lds, stream, X, ldx, M, C, g, s, chan_src, chan_depth, thr,  \
                  qmax, Xq, D, Q, magic_q, scale_out, partials, n_partials, clip_ratio, dep_table)
        if (wide_in) return halve ? OCS_LAUNCH_IN(true, uint64_t) : OCS_LAUNCH_IN(false, uint64_t);
        return halve ? OCS_LAUNCH_IN(true, uint32_t) : OCS_LAUNCH_IN(false, uint32_t);
#undef OCS_LAUNCH_IN
    }

    int un = tuning().act_un;
    if (un != 1 && un != 2 && un != 4) un = 1;
    // the prefetch looks up to 2*un strides past the item being processed
    const bool wide = tuning().act_wide > 0 || total + 2 * un * grid * kThreads >= ((int64_t)1 << 32);
    const unsigned magic = (unsigned)((((uint64_t)1) << 32) / (uint64_t)D);  // D >= 16

    hipError_t err = hipSuccess;
#define OCS_LAUNCH_EQ(H, N_, U_, I_)                                                              \
    err = launch_kernel(kTimeSplitQuantize, expand_quantize_kernel<H, N_, U_, I_>, dim3((unsigned)grid), \
                  dim3(kThreads), dep_lds, stream, X, ldx, M, C, g, s, chan_src, chan_depth, thr,  \
                  qmax, Xq, D, main_units, magic, scale_out, partials, n_partials, clip_ratio, dep_table, \
                  stepwise ? 1 : 0)
#define OCS_LAUNCH_U(H, N_, I_)                                                                   \
    do {                                                                                          \
        if (un == 4) OCS_LAUNCH_EQ(H, N_, 4, I_);                                                 \
        else if (un == 2) OCS_LAUNCH_EQ(H, N_, 2, I_);                                            \
        else OCS_LAUNCH_EQ(H, N_, 1, I_);                                                         \
    } while (0)
    if (wide) {
        if (halve) { if (nt) OCS_LAUNCH_U(true, true, uint64_t); else OCS_LAUNCH_U(true, false, uint64_t); }
        else       { if (nt) OCS_LAUNCH_U(false, true, uint64_t); else OCS_LAUNCH_U(false, false, uint64_t); }
    } else {
        if (halve) { if (nt) OCS_LAUNCH_U(true, true, uint32_t); else OCS_LAUNCH_U(true, false, uint32_t); }
        else       { if (nt) OCS_LAUNCH_U(false, true, uint32_t); else OCS_LAUNCH_U(false, false, uint32_t); }
    }
#undef OCS_LAUNCH_U
#undef OCS_LAUNCH_EQ
    return err;
}

// The weight pass with the greedy selection of Sec. 3.4 in its prologue: W2 and W3 as one launch.
// The selection needs only the column maxima (a few KB, already in memory) and a handful of
// sequential steps on them, so every workgroup repeats it for itself in LDS, behind its first
// 16-byte fetch of W, instead of waiting for a selector launch of its own: for few splits the
// repeated work (0.2 us per step on one wave) costs less than the dependent launch it replaces.
// The workgroup then expands and quantizes its share of W from the lists in LDS (Eq. 3: every
// expanded channel j is scaled by 2^-dep[j]; Eq. 1 on the grid of clip_ratio * max|W'|), with
// the arithmetic of expand_quantize_kernel.  Workgroup 0 also writes the lists, the maximum
// and the grid for the caller.  32-bit indices; C + s <= 64 << LOG2_S.
template <int LOG2_S>
__global__ __launch_bounds__(kThreads) void select_expand_quantize_kernel(
    const float* __restrict__ W, int64_t ldw, int64_t N, int C, int g, int s,
    const float* __restrict__ colmax, int32_t* __restrict__ split_src,
    int32_t* __restrict__ chan_src, int32_t* __restrict__ chan_depth, float* __restrict__ max_out,
    float clip_ratio, float qmax, float* __restrict__ scale_out, int8_t* __restrict__ Wq, int D,
    int main_units, unsigned magic) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int S = 1 << LOG2_S, P = 64 * S;
    const int E = C + s, Ke = E * g;
    float* vals = reinterpret_cast<float*>(smem);
    unsigned short* src = reinterpret_cast<unsigned short*>(vals + P);
    unsigned short* dep = src + E;
    __shared__ unsigned wred[kThreads / 64];
    const int tid = threadIdx.x;
    const bool first = blockIdx.x == 0;
    const unsigned total = (unsigned)(N * D);
    const unsigned stride = gridDim.x * kThreads;
    unsigned* __restrict__ out = reinterpret_cast<unsigned*>(Wq);

    auto fetch = [&](unsigned o, f32x4& v, unsigned& row, int& d) {
        row = 0;
        d = 0;
        if (o < total) {
            unsigned q = __umulhi(o, magic);          // floor(o / D), at most one low
            unsigned r = o - q * (unsigned)D;
            if (r >= (unsigned)D) { ++q; r -= (unsigned)D; }
            row = q;
            d = (int)r;
            if (d < main_units) v = *(reinterpret_cast<const f32x4u*>(W + (int64_t)row * ldw) + d);
        }
    };
    unsigned o = blockIdx.x * kThreads + tid;
    f32x4 cur = {}, nxt = {};
    unsigned row = 0, nrow = 0;
    int d = 0, nd = 0;
    fetch(o, cur, row, d);

    channel_maxima_to_lds(colmax, C, g, P, vals, src, dep);
    if (tid < 64) greedy_one_wave<LOG2_S>(vals, src, dep, C, s, tid, first ? split_src : nullptr);
    __syncthreads();
    unsigned m = 0;   // bit pattern of the largest entry (all entries are non-negative)
    for (int j = tid; j < E; j += kThreads) {
        if (first) {
            chan_src[j] = src[j];
            chan_depth[j] = dep[j];
        }
        const unsigned u = __float_as_uint(vals[j]);
        m = u > m ? u : m;
    }
    m = wave_umax32(m);
    if ((tid & 63) == 0) wred[tid >> 6] = m;
    __syncthreads();
    m = wred[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) m = wred[w] > m ? wred[w] : m;
    const float mx = __uint_as_float(m);
    const float T = clip_ratio * mx;
    if (first && tid == 0) {
        if (max_out) *max_out = mx;
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
    const float inv = inv_step_of(T, qmax);

    for (; o < total; o += stride) {
        fetch(o + stride, nxt, nrow, nd);
        const float* wrow = W + (int64_t)row * ldw;
        const int k = 4 * d;
        int j = k / g, t = k - j * g;
        float v[4];
        if (d < main_units) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = halved(cur[e], (int)dep[j]);
                if (++t == g) { t = 0; ++j; }
            }
        } else {
            // the four gathers are requested together and unconditionally (a column past the last
            // expanded one reads column 0 and is dropped): under a condition each would wait for
            // the one before it
            int col[4], dp[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool in = k + e < Ke;
                col[e] = in ? (int)src[in ? j : 0] * g + t : -1;
                dp[e] = in ? (int)dep[in ? j : 0] : 0;
                if (++t == g) { t = 0; ++j; }
            }
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = wrow[col[e] < 0 ? 0 : col[e]];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = col[e] >= 0 ? halved(x[e], dp[e]) : 0.0f;
        }
        out[o] = pack4(code_bits(v[0], inv, qmax), code_bits(v[1], inv, qmax),
                       code_bits(v[2], inv, qmax), code_bits(v[3], inv, qmax));
        cur = nxt;
        row = nrow;
        d = nd;
    }
}

// Whether the one-launch form serves this shape: the one-wave selector's list size, few enough
// steps for the repeated selection to be cheaper than a launch, 32-bit item indices.
bool select_expand_quantize_fits(int C, int s, int64_t N, int64_t ldq) {
    const int limit = tuning().sel_inline < 0 ? 16 : tuning().sel_inline;
    if (C + s > 1024 || s > limit || limit == 0) return false;
    return N * (ldq / 4) + 2 * 2048 * (int64_t)kThreads < ((int64_t)1 << 32);
}

hipError_t launch_select_expand_quantize(const float* W, int64_t ldw, int64_t N, int C, int g, int s,
                                         const float* colmax, int32_t* split_src, int32_t* chan_src,
                                         int32_t* chan_depth, float* max_out, float clip_ratio,
                                         float qmax, float* scale_out, int8_t* Wq, int64_t ldq,
                                         hipStream_t stream) {
    if (!select_expand_quantize_fits(C, s, N, ldq)) return hipErrorInvalidValue;
    const int E = C + s;
    const int main_units = (int)((int64_t)C * g / 4);
    const int D = (int)(ldq / 4);
    const int64_t total = N * D;
    int64_t grid = 256 * 2;   // every workgroup repeats the selection: few of them
    if (tuning().act_grid > 0) grid = tuning().act_grid;
    if (grid > ceil_div(total, kThreads)) grid = ceil_div(total, kThreads);
    const unsigned magic = (unsigned)((((uint64_t)1) << 32) / (uint64_t)D);  // D >= 16
    int log2_S = 2;        // 64 lanes x S slots hold the E entries
    while ((64 << log2_S) < E) ++log2_S;
    const unsigned lds = (unsigned)((64 << log2_S) * 4 + E * 4);
#define OCS_LAUNCH_SEQ(L_)                                                                        \
    launch_kernel(kTimeSplitQuantize, select_expand_quantize_kernel<L_>, dim3((unsigned)grid),   \
                  dim3(kThreads), lds, stream, W, ldw, N, C, g, s, colmax, split_src, chan_src,   \
                  chan_depth, max_out, clip_ratio, qmax, scale_out, Wq, D, main_units, magic)
    switch (log2_S) {
        case 2: return OCS_LAUNCH_SEQ(2);
        case 3: return OCS_LAUNCH_SEQ(3);
        default: return OCS_LAUNCH_SEQ(4);
    }
#undef OCS_LAUNCH_SEQ
}

// fp32 expanded tensor (Eq. 3 with halve != 0, the weight side of Eq. 4 with halve == 0).
// Off-line and optional: one thread per output element, coalesced stores.
__global__ __launch_bounds__(kThreads) void expand_f32_kernel(
    const float* __restrict__ T, int64_t ld, int64_t rows, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth, int halve,
    float* __restrict__ out, int64_t ldo) {
    const int Ke = (C + s) * g;
    const int64_t r = blockIdx.y;
    const float* trow = T + r * ld;
    float* orow = out + r * ldo;
    for (int k = blockIdx.x * kThreads + threadIdx.x; k < Ke; k += gridDim.x * kThreads) {
        int j = k / g, t = k - j * g;
        int src = chan_src[j];
        src = src < 0 ? 0 : (src >= C ? C - 1 : src);
        float v = trow[(int64_t)src * g + t];
        if (halve) v = halved(v, chan_depth[j]);
        orow[k] = v;
    }
}

hipError_t launch_expand_f32(const float* T, int64_t ld, int64_t rows, int C, int g, int s,
                             const int32_t* chan_src, const int32_t* chan_depth, int halve,
                             float* out, int64_t ldo, hipStream_t stream) {
    const int64_t Ke = (int64_t)(C + s) * g;
    // grid.y carries the rows (at most 65535 per launch)
    for (int64_t r0 = 0; r0 < rows; r0 += 65535) {
        int64_t nr = rows - r0 < 65535 ? rows - r0 : 65535;
        dim3 grid((unsigned)(ceil_div(Ke, kThreads) < 8 ? ceil_div(Ke, kThreads) : 8), (unsigned)nr);
        expand_f32_kernel<<<grid, kThreads, 0, stream>>>(T + r0 * ld, ld, nr, C, g, s, chan_src,
                                                         chan_depth, halve, out + r0 * ldo, ldo);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace ocs
