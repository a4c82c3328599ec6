// Greedy channel selection of Sec. 3.4 on the channel maxima.
//
// The paper splits one channel at a time, always the one that currently holds the largest
// magnitude in the layer.  Halving a channel halves its maximum exactly and its copy has the
// same maximum, so the whole sequence of choices depends only on the C channel maxima: the
// tensor itself is never re-scanned.  One workgroup keeps the (growing) list of maxima in
// LDS; each of its 256 lanes owns a block of S consecutive slots (S = 4, 8, 16 or 32, so that
// 256 * S slots hold the C + s entries; slots that do not exist yet hold -1) and caches the best
// entry of its block, so a step is one cross-lane arg-max plus a re-scan of one block by the
// lane whose slot was split: S / 4 independent 16-byte LDS reads and S compares.  Ties go to the
// lowest expanded index: the key packs the value's bit pattern (non-negative floats order like
// unsigned integers) above the complemented index.
#include "ocs_internal.h"
#include "select_lds.h"

namespace ocs {

// ONE_WAVE: up to 1024 expanded channels (most layers) are dealt over the 64 lanes of the first
// wave alone, which then runs the greedy steps by itself: no barrier and no exchange through LDS
// in a step (0.2 us instead of 0.55); the other waves help before and after.
template <int LOG2_S, bool ONE_WAVE>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const float* __restrict__ colmax, int C, int g, int s, int mode,
    const int32_t* split_in, int32_t* split_src,
    int32_t* __restrict__ chan_src, int32_t* __restrict__ chan_depth, float* __restrict__ max_out,
    float clip_ratio, float qmax, float* __restrict__ scale_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int E = C + s;
    constexpr int log2_S = LOG2_S, S = 1 << LOG2_S;
    constexpr int P = S * (ONE_WAVE ? 64 : kThreads);   // P >= E slots, the last P - E never exist
    // 4 bytes per slot and 4 per expanded channel: 8000 channels stay below the 64 KB a
    // workgroup may use without opting in to more
    float* vals = reinterpret_cast<float*>(smem);
    unsigned short* src = reinterpret_cast<unsigned short*>(vals + P);
    unsigned short* dep = src + E;
    __shared__ unsigned long long wkey[2][kThreads / 64];
    __shared__ unsigned wred[kThreads / 64];
    const int tid = threadIdx.x;

    channel_maxima_to_lds(colmax, C, g, P, vals, src, dep);

    if (mode == 0 && ONE_WAVE) {
        if (tid < 64) greedy_one_wave<LOG2_S>(vals, src, dep, C, s, tid, split_src);
        __syncthreads();
    } else if (mode == 0) {
        unsigned long long local = block_best<S>(vals, tid * S);
        // One barrier per step: the waves exchange their maxima through wkey (two sets, used
        // alternately, so that a fast wave cannot overwrite what a slow one still reads); every
        // lane then knows the step's channel and value.  The lane that owns the split slot updates
        // the list and re-scans its own block; the lane that owns the new slot folds the new entry
        // into its cached best from registers.  No lane reads a list entry another lane wrote
        // during the same step, and later reads are separated from the write by a barrier.
        for (int i = 0; i < s; ++i) {
            const int cur = C + i;
            unsigned long long k = wave_max_key(local);
            unsigned long long* wk = wkey[i & 1];
            if ((tid & 63) == 0) wk[tid >> 6] = k;
            __syncthreads();
            k = wk[0];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) k = wk[w] > k ? wk[w] : k;
            const int jstar = (int)(0xFFFFFFFFu - (unsigned)(k & 0xFFFFFFFFull));
            const float half = __uint_as_float((unsigned)(k >> 32)) * 0.5f;
            const bool owns_old = (jstar >> log2_S) == tid;
            const bool owns_new = (cur >> log2_S) == tid;
            if (owns_old) {
                vals[jstar] = half;
                unsigned short d = (unsigned short)(dep[jstar] + 1);
                dep[jstar] = d;
                vals[cur] = half;
                src[cur] = src[jstar];
                dep[cur] = d;
                split_src[i] = jstar;
                local = block_best<S>(vals, tid * S);   // sees the new slot too, if it is this lane's
            } else if (owns_new) {
                const unsigned long long kn = key_of_bits(__float_as_uint(half), cur);
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

    unsigned m = 0;   // bit pattern of the largest entry (all entries are non-negative)
    for (int j = tid; j < E; j += kThreads) {
        chan_src[j] = src[j];
        chan_depth[j] = dep[j];
        const unsigned u = __float_as_uint(vals[j]);
        m = u > m ? u : m;
    }
    m = wave_umax32(m);
    if ((tid & 63) == 0) wred[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) m = wred[w] > m ? wred[w] : m;
        const float mx = __uint_as_float(m);
        if (max_out) *max_out = mx;
        if (scale_out) {
            float T = clip_ratio * mx;
            scale_out[0] = T;
            scale_out[1] = T / qmax;
        }
    }
}

hipError_t launch_select(const float* colmax, int C, int g, int s, int mode,
                         const int32_t* split_in, int32_t* split_src, int32_t* chan_src,
                         int32_t* chan_depth, float* max_out, float clip_ratio, float qmax,
                         float* scale_out, hipStream_t stream) {
    const int E = C + s;   // E <= kMaxExpanded is checked by the caller
    const bool one_wave = E <= 1024;
    const int lanes = one_wave ? 64 : kThreads;
    int log2_S = 2;        // lanes x S slots hold the E entries
    while ((lanes << log2_S) < E) ++log2_S;
    if (log2_S > 5) return hipErrorInvalidValue;
    const size_t lds = (size_t)(lanes << log2_S) * 4 + (size_t)E * 4;
#define OCS_SELECT(L_, W_)                                                                         \
    select_kernel<L_, W_><<<1, kThreads, lds, stream>>>(colmax, C, g, s, mode, split_in, split_src, \
                                                        chan_src, chan_depth, max_out, clip_ratio, \
                                                        qmax, scale_out)
    if (one_wave) {
        switch (log2_S) {
            case 2: OCS_SELECT(2, true); break;
            case 3: OCS_SELECT(3, true); break;
            default: OCS_SELECT(4, true); break;
        }
    } else {
        switch (log2_S) {
            case 2: OCS_SELECT(2, false); break;
            case 3: OCS_SELECT(3, false); break;
            case 4: OCS_SELECT(4, false); break;
            default: OCS_SELECT(5, false); break;
        }
    }
#undef OCS_SELECT
    return hipGetLastError();
}

}  // namespace ocs
