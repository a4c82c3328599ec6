// Measurement helpers: plain kernels of known work that put this chip's own ceilings beside the
// kernels of the path (no passage of the paper).  A copy, a read-only sweep and a fill of known
// size for the memory system; the same read over a buffer small enough to stay in every L2 for the
// path between the L2s and the compute units; a bare loop of the matrix instruction the GEMM uses,
// on whatever operand bytes the caller supplies (constant or random: the clock under matrix load
// depends on how many bits toggle).  None of them is called by the path itself.
#include "ocs_internal.h"

namespace ocs {

// Plain device-to-device copy with 16-byte accesses.
__global__ __launch_bounds__(kThreads) void calib_copy_kernel(const f32x4* __restrict__ src,
                                                              f32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// The same work with no loop: one 16-byte group per lane, one workgroup per 4 KB, handed out in
// order by the dispatcher (workgroups == 0 in the calls below selects this form).
__global__ __launch_bounds__(kThreads) void calib_copy_shot_kernel(const f32x4* __restrict__ src,
                                                                   f32x4* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

static unsigned shot_grid(size_t n16) { return (unsigned)((n16 + kThreads - 1) / kThreads); }

hipError_t launch_calib_copy(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t stream) {
    if (workgroups == 0)
        calib_copy_shot_kernel<<<shot_grid(bytes / 16), kThreads, 0, stream>>>(static_cast<const f32x4*>(src),
                                                                               static_cast<f32x4*>(dst), bytes / 16);
    else
        calib_copy_kernel<<<(unsigned)workgroups, kThreads, 0, stream>>>(static_cast<const f32x4*>(src),
                                                                         static_cast<f32x4*>(dst), bytes / 16);
    return hipGetLastError();
}

// The split+quantize pass's traffic pattern without its arithmetic: 16 bytes read and 4 written per
// lane (the low byte of each of the four words), in the one-shot form or as a grid-stride loop.
__device__ __forceinline__ unsigned low_bytes(const i32x4& v) {
    return ((unsigned)v[0] & 0xFFu) | (((unsigned)v[1] & 0xFFu) << 8) | (((unsigned)v[2] & 0xFFu) << 16) |
           ((unsigned)v[3] << 24);
}
__global__ __launch_bounds__(kThreads) void calib_pack_shot_kernel(const i32x4* __restrict__ src,
                                                                   unsigned* __restrict__ dst, size_t n16) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n16) dst[i] = low_bytes(src[i]);
}
__global__ __launch_bounds__(kThreads) void calib_pack_kernel(const i32x4* __restrict__ src,
                                                              unsigned* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride) dst[i] = low_bytes(src[i]);
}

hipError_t launch_calib_pack(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t stream) {
    if (workgroups == 0)
        calib_pack_shot_kernel<<<shot_grid(bytes / 16), kThreads, 0, stream>>>(static_cast<const i32x4*>(src),
                                                                               static_cast<unsigned*>(dst), bytes / 16);
    else
        calib_pack_kernel<<<(unsigned)workgroups, kThreads, 0, stream>>>(static_cast<const i32x4*>(src),
                                                                         static_cast<unsigned*>(dst), bytes / 16);
    return hipGetLastError();
}

// Read-only sweep: n16 * passes 16-byte loads as one flat grid-stride stream over the n16 groups of
// src (with passes > 1 the stream wraps around: n16 is then a power of two), two loads in flight
// per lane.  A buffer far larger than the caches with one pass gives the HBM read rate; a buffer
// of a megabyte or two with many passes stays in every L2, and the rate is then that at which the
// compute units draw from their L2s.  The values are folded into one word per lane and compared
// with a value they practically never take, so that the loads cannot be dropped.
__global__ __launch_bounds__(kThreads) void calib_read_kernel(const i32x4* __restrict__ src, size_t n16,
                                                              size_t items, size_t mask,
                                                              int* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    int acc = 0;
    for (; i + stride < items; i += 2 * stride) {
        const i32x4 a = src[i & mask], b = src[(i + stride) & mask];
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3];
    }
    if (i < items) {
        const i32x4 a = src[i & mask];
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    if (acc == 0x5a5a1234) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(kThreads) void calib_read_shot_kernel(const i32x4* __restrict__ src, size_t n16,
                                                                   int* __restrict__ sink) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n16) return;
    const i32x4 a = src[i];
    if ((a[0] ^ a[1] ^ a[2] ^ a[3]) == 0x5a5a1234) sink[0] = 1;
}

hipError_t launch_calib_read(const void* src, size_t bytes, int passes, int workgroups, void* sink,
                             hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (workgroups == 0) {     // one pass, one-shot form
        calib_read_shot_kernel<<<shot_grid(n16), kThreads, 0, stream>>>(static_cast<const i32x4*>(src), n16,
                                                                        static_cast<int*>(sink));
        return hipGetLastError();
    }
    // one pass: no wrap (mask of all ones); several: n16 is a power of two and the index wraps
    const size_t mask = passes > 1 ? n16 - 1 : ~(size_t)0;
    calib_read_kernel<<<(unsigned)workgroups, kThreads, 0, stream>>>(static_cast<const i32x4*>(src), n16,
                                                                     n16 * (size_t)passes, mask,
                                                                     static_cast<int*>(sink));
    return hipGetLastError();
}

// Fill with 16-byte stores, plain or with the streaming (non-temporal) hint.
template <bool NT>
__global__ __launch_bounds__(kThreads) void calib_fill_kernel(i32x4* __restrict__ dst, size_t n16, int value) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    const i32x4 v = {value, value, value, value};
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride) {
        if (NT) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void calib_fill_shot_kernel(i32x4* __restrict__ dst, size_t n16, int value) {
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const i32x4 v = {value, value, value, value};
    if (i < n16) {
        if (NT) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

hipError_t launch_calib_fill(void* dst, size_t bytes, int value, int nontemporal, int workgroups,
                             hipStream_t stream) {
    if (workgroups == 0) {
        const unsigned sg = shot_grid(bytes / 16);
        if (nontemporal)
            calib_fill_shot_kernel<true><<<sg, kThreads, 0, stream>>>(static_cast<i32x4*>(dst), bytes / 16, value);
        else
            calib_fill_shot_kernel<false><<<sg, kThreads, 0, stream>>>(static_cast<i32x4*>(dst), bytes / 16, value);
        return hipGetLastError();
    }
    const unsigned g = (unsigned)workgroups;
    if (nontemporal)
        calib_fill_kernel<true><<<g, kThreads, 0, stream>>>(static_cast<i32x4*>(dst), bytes / 16, value);
    else
        calib_fill_kernel<false><<<g, kThreads, 0, stream>>>(static_cast<i32x4*>(dst), bytes / 16, value);
    return hipGetLastError();
}

// Bare matrix-core loop: every wave holds two A and two B fragments (16 bytes per lane each, taken
// from `operands`, 16 KB) and issues `iters` rounds of the four v_mfma_i32_32x32x32_i8 that pair
// them, on four independent accumulators: no memory access and no LDS inside the loop.  A launch
// performs workgroups * 4 waves * iters * 4 * 65536 integer operations.
__global__ __launch_bounds__(kThreads) void calib_mfma_kernel(const i32x4* __restrict__ operands, int iters,
                                                              int* __restrict__ sink) {
    const int t = threadIdx.x;
    const i32x4 a0 = operands[t], b0 = operands[256 + t], a1 = operands[512 + t], b1 = operands[768 + t];
    i32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b0, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b1, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, c3, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int v = 0; v < 16; ++v) s ^= c0[v] ^ c1[v] ^ c2[v] ^ c3[v];
    sink[(size_t)blockIdx.x * kThreads + t] = s;
}

hipError_t launch_calib_mfma(const void* operands, int iters, int workgroups, void* sink, hipStream_t stream) {
    calib_mfma_kernel<<<(unsigned)workgroups, kThreads, 0, stream>>>(static_cast<const i32x4*>(operands), iters,
                                                                     static_cast<int*>(sink));
    return hipGetLastError();
}

}  // namespace ocs
