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
#include "ocs_internal.h"

namespace ocs {

// One value onto the grid: one fp32 multiply by qmax/T, round half to even, saturate.
__device__ __forceinline__ int code_of(float v, float inv_step, float qmax) {
    float r = __builtin_rintf(v * inv_step);
    r = __builtin_fminf(__builtin_fmaxf(r, -qmax), qmax);
    return (int)r;
}

__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d) {
    return (unsigned)(a & 0xFF) | ((unsigned)(b & 0xFF) << 8) | ((unsigned)(c & 0xFF) << 16) |
           ((unsigned)d << 24);
}

// qmax / T as one correctly rounded division, kept finite so that 0 * inv_step stays 0.
__device__ __forceinline__ float inv_step_of(float T, float qmax) {
    if (!(T > 0.0f)) return 0.0f;
    return __builtin_fminf(__fdiv_rn(qmax, T), 3.402823466e+38f);
}

// Workgroup (TX, TY): TY rows at a time, lane tx walks the packed dwords of a row with
// stride TX.  main_units = number of leading dwords whose four inputs are the contiguous,
// 16-byte aligned X[r, 4d .. 4d+3] (0 when X does not allow vector loads).
template <bool HALVE>
__global__ __launch_bounds__(kThreads) void expand_quantize_kernel(
    const float* __restrict__ X, int64_t ldx, int64_t M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth,
    const float* thr, float qmax, int8_t* __restrict__ Xq, int64_t ldq, int main_units,
    int rows_per_block, float* scale_out) {
    const int tx = threadIdx.x, ty = threadIdx.y, TX = blockDim.x, TY = blockDim.y;
    const float T = *thr;
    const float inv = inv_step_of(T, qmax);
    if (scale_out != nullptr && blockIdx.x == 0 && tx == 0 && ty == 0) {
        scale_out[0] = T;
        scale_out[1] = T / qmax;
    }
    const int D = (int)(ldq >> 2);
    const int Ke = (C + s) * g;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > M) r1 = M;

    for (int64_t r = r0 + ty; r < r1; r += TY) {
        const float* xrow = X + r * ldx;
        unsigned* qrow = reinterpret_cast<unsigned*>(Xq + r * ldq);

        // identity region: columns below C*g sit where they were
#pragma unroll 4
        for (int d = tx; d < main_units; d += TX) {
            f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xrow) + d);
            if (HALVE) {
                int j = (4 * d) / g, t = 4 * d - j * g;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = v[e] * ldexpf(1.0f, -chan_depth[j]);
                    if (++t == g) { t = 0; ++j; }
                }
            }
            qrow[d] = pack4(code_of(v[0], inv, qmax), code_of(v[1], inv, qmax),
                            code_of(v[2], inv, qmax), code_of(v[3], inv, qmax));
        }

        // gather region: leftover columns, the appended channels, and the zero padding
        for (int d = main_units + tx; d < D; d += TX) {
            int code[4];
            int k = 4 * d;
            int j = k / g, t = k - j * g;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int c = 0;
                if (k + e < Ke) {
                    int src = chan_src ? chan_src[j] : j;
                    src = src < 0 ? 0 : (src >= C ? C - 1 : src);
                    float v = xrow[(int64_t)src * g + t];
                    if (HALVE) v = v * ldexpf(1.0f, -chan_depth[j]);
                    c = code_of(v, inv, qmax);
                }
                code[e] = c;
                if (++t == g) { t = 0; ++j; }
            }
            qrow[d] = pack4(code[0], code[1], code[2], code[3]);
        }
    }
}

hipError_t launch_expand_quantize(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                  const int32_t* chan_src, const int32_t* chan_depth,
                                  const float* thr, float qmax, int8_t* Xq, int64_t ldq,
                                  float* scale_out, hipStream_t stream) {
    const int64_t K = (int64_t)C * g;
    bool vec_ok = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 4 == 0);
    int main_units = vec_ok ? (int)(K / 4) : 0;
    const int D = (int)(ldq / 4);

    // lanes along the row: the power of two in {16, 32, 64} that wastes the fewest lanes
    int tx = 64;
    int64_t best = -1;
    for (int cand = 64; cand >= 16; cand >>= 1) {
        int64_t padded = ceil_div(D, cand) * cand;
        if (best < 0 || padded < best) { best = padded; tx = cand; }
    }
    if (tuning().act_tx > 0) tx = tuning().act_tx;
    const int ty = kThreads / tx;

    // rows per workgroup: a few passes over TY rows, and enough workgroups to fill the chip
    int64_t rpb = (int64_t)ty * 2;
    while (rpb > ty && ceil_div(M, rpb) < 2048) rpb -= ty;
    if (tuning().act_rows_per_block > 0) rpb = tuning().act_rows_per_block;
    const int64_t blocks = ceil_div(M, rpb);

    dim3 block(tx, ty);
    if (chan_depth != nullptr)
        expand_quantize_kernel<true><<<(unsigned)blocks, block, 0, stream>>>(
            X, ldx, M, C, g, s, chan_src, chan_depth, thr, qmax, Xq, ldq, main_units, (int)rpb,
            scale_out);
    else
        expand_quantize_kernel<false><<<(unsigned)blocks, block, 0, stream>>>(
            X, ldx, M, C, g, s, chan_src, chan_depth, thr, qmax, Xq, ldq, main_units, (int)rpb,
            scale_out);
    return hipGetLastError();
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
        if (halve) v = v * ldexpf(1.0f, -chan_depth[j]);
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
