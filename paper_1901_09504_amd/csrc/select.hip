// Greedy channel selection of Sec. 3.4 on the channel maxima.
//
// The paper splits one channel at a time, always the one that currently holds the largest
// magnitude in the layer.  Halving a channel halves its maximum exactly and its copy has the
// same maximum, so the whole sequence of choices depends only on the C channel maxima: the
// tensor itself is never re-scanned.  One workgroup keeps the (growing) list of maxima in
// LDS; each of its 256 lanes caches the best entry among the slots it owns (slot j belongs to
// lane j mod 256), so a step is one cross-lane arg-max plus a re-scan by the at most two lanes
// whose slots changed.  Ties go to the lowest expanded index: the key packs the value's bit
// pattern (non-negative floats order like unsigned integers) above the complemented index.
#include "ocs_internal.h"

namespace ocs {

__device__ inline unsigned long long key_of(float v, int j) {
    return ((unsigned long long)__float_as_uint(v) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)j);
}

// Largest key of the wave: largest value first, then (through the complemented index in the
// low word) the lowest index among the lanes that hold it.
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long k) {
    const unsigned hi = (unsigned)(k >> 32), lo = (unsigned)k;
    const unsigned mhi = wave_umax32(hi);
    const unsigned mlo = wave_umax32(hi == mhi ? lo : 0u);
    return ((unsigned long long)mhi << 32) | mlo;
}

__global__ __launch_bounds__(kThreads) void select_kernel(
    const float* __restrict__ colmax, int C, int g, int s, int mode,
    const int32_t* split_in, int32_t* split_src,
    int32_t* __restrict__ chan_src, int32_t* __restrict__ chan_depth, float* __restrict__ max_out,
    float clip_ratio, float qmax, float* __restrict__ scale_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int E = C + s;
    // 8 bytes per expanded channel: 8000 channels stay below the 64 KB a workgroup may use
    // without opting in to more
    float* vals = reinterpret_cast<float*>(smem);
    unsigned short* src = reinterpret_cast<unsigned short*>(vals + E);
    unsigned short* dep = src + E;
    __shared__ unsigned long long wkey[2][kThreads / 64];
    __shared__ float red[kThreads];
    const int tid = threadIdx.x;

    // channel maxima: one coalesced, independent load per column, folded per channel with LDS
    // atomics on the bit pattern (non-negative floats order like unsigned integers)
    for (int j = tid; j < C; j += kThreads) {
        vals[j] = 0.0f;
        src[j] = (unsigned short)j;
        dep[j] = 0;
    }
    __syncthreads();
    {
        const int K = C * g;
        unsigned* vbits = reinterpret_cast<unsigned*>(vals);
#pragma unroll 8
        for (int k = tid; k < K; k += kThreads)
            atomicMax(&vbits[k / g], __float_as_uint(colmax[k]));
    }
    __syncthreads();

    if (mode == 0) {
        unsigned long long local = 0;
        for (int j = tid; j < C; j += kThreads) {
            unsigned long long k = key_of(vals[j], j);
            local = k > local ? k : local;
        }
        // One barrier per step: the waves exchange their maxima through wkey (two sets, used
        // alternately, so that a fast wave cannot overwrite what a slow one still reads); every
        // lane then knows the step's channel and value.  The lane that owns the split slot updates
        // the list and re-scans its own slots; the lane that owns the new slot folds the new entry
        // into its cached best from registers.  No lane reads a list entry another lane wrote
        // during the same step, and later reads are separated from the write by a barrier.
        for (int i = 0; i < s; ++i) {
            const int cur = C + i;
            unsigned long long k = wave_max_u64(local);
            unsigned long long* wk = wkey[i & 1];
            if ((tid & 63) == 0) wk[tid >> 6] = k;
            __syncthreads();
            k = wk[0];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) k = wk[w] > k ? wk[w] : k;
            const int jstar = (int)(0xFFFFFFFFu - (unsigned)(k & 0xFFFFFFFFull));
            const float half = __uint_as_float((unsigned)(k >> 32)) * 0.5f;
            const bool owns_old = (jstar % kThreads) == tid;
            const bool owns_new = (cur % kThreads) == tid;
            if (owns_old) {
                vals[jstar] = half;
                unsigned short d = (unsigned short)(dep[jstar] + 1);
                dep[jstar] = d;
                vals[cur] = half;
                src[cur] = src[jstar];
                dep[cur] = d;
                split_src[i] = jstar;
                // re-scan of this lane's slots (the new slot too, if it is this lane's): four
                // independent LDS reads per trip, so their latencies overlap
                unsigned long long l0 = 0, l1 = 0, l2 = 0, l3 = 0;
                int j = tid;
                for (; j + 3 * kThreads <= cur; j += 4 * kThreads) {
                    const float v0 = vals[j], v1 = vals[j + kThreads], v2 = vals[j + 2 * kThreads],
                                v3 = vals[j + 3 * kThreads];
                    const unsigned long long k0 = key_of(v0, j), k1 = key_of(v1, j + kThreads),
                                             k2 = key_of(v2, j + 2 * kThreads),
                                             k3 = key_of(v3, j + 3 * kThreads);
                    l0 = k0 > l0 ? k0 : l0;
                    l1 = k1 > l1 ? k1 : l1;
                    l2 = k2 > l2 ? k2 : l2;
                    l3 = k3 > l3 ? k3 : l3;
                }
                for (; j <= cur; j += kThreads) {
                    const unsigned long long kk = key_of(vals[j], j);
                    l0 = kk > l0 ? kk : l0;
                }
                l0 = l0 > l1 ? l0 : l1;
                l2 = l2 > l3 ? l2 : l3;
                local = l0 > l2 ? l0 : l2;
            } else if (owns_new) {
                const unsigned long long kn = key_of(half, cur);
                local = kn > local ? kn : local;
            }
        }
        __syncthreads();
    } else {
        if (tid == 0) {
            for (int i = 0; i < s; ++i) {
                const int cur = C + i;
                int j = split_in[i];
                j = j < 0 ? 0 : (j >= cur ? cur - 1 : j);
                unsigned short d = (unsigned short)(dep[j] + 1);
                dep[j] = d;
                vals[cur] = vals[j];  // copies are not halved: the maximum stays
                src[cur] = src[j];
                dep[cur] = d;
            }
        }
    }
    __syncthreads();

    float m = 0.0f;
    for (int j = tid; j < E; j += kThreads) {
        chan_src[j] = src[j];
        chan_depth[j] = dep[j];
        m = fmaxf(m, vals[j]);
    }
    red[tid] = m;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (tid < w) red[tid] = fmaxf(red[tid], red[tid + w]);
        __syncthreads();
    }
    if (tid == 0) {
        if (max_out) *max_out = red[0];
        if (scale_out) {
            float T = clip_ratio * red[0];
            scale_out[0] = T;
            scale_out[1] = T / qmax;
        }
    }
}

hipError_t launch_select(const float* colmax, int C, int g, int s, int mode,
                         const int32_t* split_in, int32_t* split_src, int32_t* chan_src,
                         int32_t* chan_depth, float* max_out, float clip_ratio, float qmax,
                         float* scale_out, hipStream_t stream) {
    size_t lds = (size_t)(C + s) * 8;  // C + s <= kMaxExpanded is checked by the caller
    select_kernel<<<1, kThreads, lds, stream>>>(colmax, C, g, s, mode, split_in, split_src,
                                                chan_src, chan_depth, max_out, clip_ratio, qmax,
                                                scale_out);
    return hipGetLastError();
}

}  // namespace ocs
