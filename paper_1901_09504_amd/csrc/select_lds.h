// Device-side pieces of the greedy channel selection of Sec. 3.4, shared by the selector kernel
// and by the weight pass that runs the selection in its own prologue.
//
// The list of channel maxima lives in LDS: `vals` holds P = lanes * S slots (slots that do not
// exist yet hold -1.0), `src` and `dep` the original channel and the number of halvings of each
// of the C + s expanded channels.  Every lane owns a block of S consecutive slots and caches the
// best entry of its block.  Ties go to the lowest expanded index: the key packs the value's bit
// pattern (non-negative floats order like unsigned integers) above the complemented index.
#pragma once
#include "ocs_internal.h"

namespace ocs {

__device__ inline unsigned long long key_of_bits(unsigned bits, int j) {
    return ((unsigned long long)bits << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)j);
}

// Largest key of the wave: largest value first, then the lowest index among the lanes that hold
// it.  One reduction, on the values alone: blocks lie in lane order and every lane caches the
// lowest slot among the equals of its own block, so among the lanes that hold the largest value the
// lowest lane holds the lowest index (lanes without entries carry key 0 and sit above all lanes
// of the list that have some).
__device__ __forceinline__ unsigned long long wave_max_key(unsigned long long k) {
    const unsigned hi = (unsigned)(k >> 32);
    const unsigned mhi = wave_umax32(hi);
    const int winner = __ffsll((long long)__ballot(hi == mhi)) - 1;
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)k, winner);
    return ((unsigned long long)mhi << 32) | lo;
}

// Best entry of a block of S slots held in registers (v[q][e] = slot j0 + 4q + e): the largest
// value, the lowest slot among equals (slots are visited in ascending order and only a strictly
// larger value replaces the best so far).  Values are compared as signed integers on their bit
// patterns: existing entries are non-negative floats, slots that do not exist yet hold -1.0
// (negative as an integer) and can never win.  0 when the block holds no entry.
template <int S>
__device__ __forceinline__ unsigned long long best_of(const f32x4 (&v)[S / 4], int j0) {
    int bv = -1, bj = 0;
#pragma unroll
    for (int q = 0; q < S / 4; ++q) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int u = (int)__float_as_uint(v[q][e]);
            const bool better = u > bv;
            bv = better ? u : bv;
            bj = better ? 4 * q + e : bj;
        }
    }
    return bv < 0 ? 0ull : key_of_bits((unsigned)bv, j0 + bj);
}

// The block of S slots that starts at slot j0, read from LDS (all reads issued together), and
// its best entry.
template <int S>
__device__ __forceinline__ void block_load(const float* vals, int j0, f32x4 (&v)[S / 4]) {
    const f32x4* p = reinterpret_cast<const f32x4*>(vals + j0);
#pragma unroll
    for (int q = 0; q < S / 4; ++q) v[q] = p[q];
}
template <int S>
__device__ __forceinline__ unsigned long long block_best(const float* vals, int j0) {
    f32x4 v[S / 4];
    block_load<S>(vals, j0, v);
    return best_of<S>(v, j0);
}

// Channel maxima from the K = C * g column maxima into vals[0 .. C), the other slots marked as
// not existing, src/dep set to the identity.  One coalesced, independent load per column, folded
// per channel with LDS atomics on the bit pattern.  Called by all kThreads lanes of the
// workgroup; contains barriers, and ends with one.
__device__ __forceinline__ void channel_maxima_to_lds(const float* __restrict__ colmax, int C, int g,
                                                      int P, float* vals, unsigned short* src,
                                                      unsigned short* dep) {
    const int tid = threadIdx.x;
    for (int j = tid; j < P; j += kThreads) vals[j] = j < C ? 0.0f : -1.0f;
    for (int j = tid; j < C; j += kThreads) {
        src[j] = (unsigned short)j;
        dep[j] = 0;
    }
    __syncthreads();
    const int K = C * g;
    unsigned* vbits = reinterpret_cast<unsigned*>(vals);
    // Sixteen loads per lane are requested before the first value is used: the column maxima were
    // written a moment ago by other CUs and every load waits a whole trip through the fabric.  (The
    // compiler keeps a load behind the LDS atomic that precedes it in program order, so a plain
    // loop, unrolled or not, made one trip per column of a lane: most of the selector's time.)
    constexpr int UN = 16;
    for (int k0 = tid; k0 < K; k0 += UN * kThreads) {
        float v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + u * kThreads;
            v[u] = colmax[k < K ? k : K - 1];
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + u * kThreads;
            if (k < K) atomicMax(&vbits[k / g], __float_as_uint(v[u]));
        }
    }
    __syncthreads();
}

// The s greedy steps on a list of at most 64 * S entries, run by the 64 lanes of ONE wave (lane
// = its index in the wave, which owns slots lane*S ...): no barrier and no exchange through LDS
// in a step.  A wave's LDS accesses execute in program order: a slot written in one step is seen
// by whichever lane re-scans its block in a later one.  split_src (may be null) receives the
// expanded index chosen at every step.
template <int LOG2_S>
__device__ __forceinline__ void greedy_one_wave(float* vals, unsigned short* src, unsigned short* dep,
                                                int C, int s, int lane, int32_t* split_src) {
    constexpr int S = 1 << LOG2_S;
    unsigned long long local = block_best<S>(vals, lane * S);
    for (int i = 0; i < s; ++i) {
        const int cur = C + i;
        const unsigned long long k = wave_max_key(local);   // lane 0 always has an entry
        const int jstar = (int)(0xFFFFFFFFu - (unsigned)(k & 0xFFFFFFFFull));
        const float half = __uint_as_float((unsigned)(k >> 32)) * 0.5f;
        if ((jstar >> LOG2_S) == lane) {
            // both look-ups first (one trip to LDS for the two), then the stores, then the re-scan
            const unsigned short s0 = src[jstar];
            const unsigned short d = (unsigned short)(dep[jstar] + 1);
            vals[jstar] = half;
            vals[cur] = half;
            dep[jstar] = d;
            src[cur] = s0;
            dep[cur] = d;
            if (split_src) split_src[i] = jstar;
            local = block_best<S>(vals, lane * S);
        } else if ((cur >> LOG2_S) == lane) {
            const unsigned long long kn = key_of_bits(__float_as_uint(half), cur);
            local = kn > local ? kn : local;
        }
    }
}

}  // namespace ocs
