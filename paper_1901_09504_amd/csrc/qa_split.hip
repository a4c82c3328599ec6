// Quantization-aware splitting of the weights (Sec. 3.3), off-line.
//
// In units of the grid step a QA split replaces w by the pair ((w - 1/2)/2, (w + 1/2)/2);
// rounded with that section's Q(x) = floor(x + 1/2) the two members add up to Q(w).  The
// channels to split and the threshold are those of the plain-halving procedure (Sec. 3.4,
// Eq. 3) on the same tensor, which fixes the step before any QA pair is formed; the channel
// that keeps its index takes the "-" member, the appended copy the "+" member.  An expanded
// channel is therefore its source channel pushed through its own short history of members
// (chan_path, one bit per split, first split in bit 0), one fp32 add/subtract and one exact
// halving per split, in the order the splits happened.
#include "ocs_internal.h"

namespace ocs {

// Histories of the expanded channels from the split list.  The list is short and strictly
// sequential (a split's parent may itself be a copy made a step earlier): one lane replays it
// in LDS, then the workgroup writes the result out.
__global__ __launch_bounds__(kThreads) void qa_paths_kernel(const int32_t* __restrict__ split_src,
                                                            int C, int s,
                                                            uint32_t* __restrict__ chan_path, int staged) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int E = C + s;
    uint32_t* path = reinterpret_cast<uint32_t*>(smem);
    // the split list is staged in LDS when it fits beside the histories: the replay below is
    // one dependent chain, and a global load per step would be most of it
    int32_t* list = reinterpret_cast<int32_t*>(path + E);
    unsigned char* len = reinterpret_cast<unsigned char*>(list + (staged ? s : 0));
    for (int j = threadIdx.x; j < E; j += kThreads) {
        path[j] = 0u;
        len[j] = 0;
    }
    if (staged)
        for (int i = threadIdx.x; i < s; i += kThreads) list[i] = split_src[i];
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 0; i < s; ++i) {
            const int cur = C + i;
            int p = staged ? list[i] : split_src[i];
            p = p < 0 ? 0 : (p >= cur ? cur - 1 : p);
            const unsigned l = len[p] < 31 ? len[p] : 31;   // a history grows like log2(s): never 31
            path[cur] = path[p] | (1u << l);
            len[p] = (unsigned char)(l + 1);
            len[cur] = (unsigned char)(l + 1);
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < E; j += kThreads) chan_path[j] = path[j];
}

// One lane per packed dword of codes (four expanded columns of one row).  Which dwords of a row
// touch a split or an appended channel does not depend on the row; each workgroup works that out
// once (a bit per dword, the list of the dwords concerned and, per listed element, its source
// column, history and depth, all in LDS).  The work then falls into two passes over disjoint
// dwords: the plain ones (nearly all: r is a few percent) as one flat range with a grid stride,
// one 16-byte load and four roundings each, the next item's load requested before this one is
// rounded; and the listed dwords of every row, every lane busy with the element-by-element replay
// of histories on four gathered values.  Mixed in one pass, a single listed dword in a wave made
// all 64 lanes wait through the replay code, which nearly every wave had to; and any second
// memory access inside the streaming loop made the compiler wait for every outstanding request
// before each use.
constexpr int kQaMaskDwords = 32768;   // rows of up to 128 KB of codes take the two-pass route
constexpr int kQaListCap = 4096;       // listed (not plain) dwords per row it can hold
constexpr int kQaMetaCap = 1024;       // listed dwords whose per-element source, history and depth fit in LDS

// the element-by-element member: source value through its channel's history, fp32 out if wanted
__device__ __forceinline__ unsigned qa_dword_generic(
    const float* __restrict__ W, int64_t ldw, int64_t n, int d, int C, int g, int Ke,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth,
    const uint32_t* __restrict__ chan_path, float half_step, float inv, float qmax,
    float* __restrict__ W_out, int64_t ldo) {
    unsigned packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int k = 4 * d + e;
        int code = 0;
        if (k < Ke) {
            const int j = k / g, t = k - j * g;
            int src = chan_src[j];
            src = src < 0 ? 0 : (src >= C ? C - 1 : src);
            float x = W[n * ldw + (int64_t)src * g + t];
            const int depth = chan_depth[j] < 31 ? chan_depth[j] : 31;
            const uint32_t path = chan_path[j];
            for (int b = 0; b < depth; ++b) {
                const float m = ((path >> b) & 1u) ? x + half_step : x - half_step;
                x = m * 0.5f;
            }
            if (W_out) W_out[n * ldo + k] = x;
            float p = x * inv;
            p = __builtin_amdgcn_fmed3f(p, -qmax, qmax);
            code = (int)floorf(p + 0.5f);        // Sec. 3.3's Q(x) = floor(x + 1/2)
        }
        packed |= ((unsigned)code & 0xFFu) << (8 * e);
    }
    return packed;
}

template <typename Index>
__global__ __launch_bounds__(kThreads) void expand_quantize_qa_kernel(
    const float* __restrict__ W, int64_t ldw, int64_t N, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const int32_t* __restrict__ chan_depth,
    const uint32_t* __restrict__ chan_path, const float* __restrict__ thr, float* __restrict__ scale_out,
    float qmax, float* __restrict__ W_out, int64_t ldo, int8_t* __restrict__ Wq, int D, unsigned magic,
    int meta_cap, int side_wgs) {
    // per element of the listed dwords (row-independent): source column (-1: past the last
    // expanded column), history bits, depth; meta_cap dwords' worth, sized by the launcher
    extern __shared__ __align__(16) unsigned char qa_meta[];
    int* meta_col = reinterpret_cast<int*>(qa_meta);
    uint32_t* meta_path = reinterpret_cast<uint32_t*>(meta_col + 4 * meta_cap);
    unsigned char* meta_dep = reinterpret_cast<unsigned char*>(meta_path + 4 * meta_cap);
    __shared__ unsigned plain_mask[kQaMaskDwords / 32];
    __shared__ unsigned short listed[kQaListCap];
    __shared__ unsigned short plain_before[kQaMaskDwords / 32];   // plain dwords in the words before
    __shared__ int n_listed;
    __shared__ unsigned chan_split[(kMaxExpanded + 31) / 32];   // bit j: channel j < C was split
    const int Ke = (C + s) * g;
    const int Dk = (Ke + 3) / 4;   // dwords that hold expanded columns; the rest of a row is zero padding
    // two passes only when codes alone are wanted and a row's dwords fit the mask
    const bool two_pass = W_out == nullptr && Wq != nullptr && D <= kQaMaskDwords;
    if (two_pass) {
        const int words = (D + 31) / 32;
        for (int w = threadIdx.x; w < words; w += kThreads) plain_mask[w] = 0u;
        for (int w = threadIdx.x; w < (C + 31) / 32; w += kThreads) chan_split[w] = 0u;
        __syncthreads();
        // which channels were split (or are not their own source): one round of independent loads,
        // so that the dword test below reads LDS only (as a chain of look-ups in global memory per
        // dword this set-up was most of the kernel's time on small split counts)
        for (int j = threadIdx.x; j < C; j += kThreads)
            if (chan_depth[j] != 0 || chan_src[j] != j) atomicOr(&chan_split[j >> 5], 1u << (j & 31));
        __syncthreads();
        for (int d = threadIdx.x; d < D; d += kThreads) {
            bool plain = 4 * d + 3 < C * g;   // inside the identity region ...
            if (plain) {
                const int j0 = (4 * d) / g, j1 = (4 * d + 3) / g;   // ... and no channel of it split
                for (int j = j0; j <= j1; ++j) plain = plain && !((chan_split[j >> 5] >> (j & 31)) & 1u);
            }
            if (plain) atomicOr(&plain_mask[d >> 5], 1u << (d & 31));
        }
        __syncthreads();
        // The list must be the same in every workgroup (pass 2 deals (row, list entry) pairs over
        // the whole grid): a listed dword's place is its rank among the listed ones.
        if (threadIdx.x == 0) {
            int before = 0;
            for (int w = 0; w < words; ++w) {
                plain_before[w] = (unsigned short)before;
                before += __popc(plain_mask[w]);
            }
            n_listed = Dk - before;      // every plain dword lies below Dk; padding dwords are not listed
        }
        __syncthreads();
        for (int d = threadIdx.x; d < Dk; d += kThreads) {
            const unsigned m = plain_mask[d >> 5];
            if (!((m >> (d & 31)) & 1u)) {
                const int rank = d - (int)plain_before[d >> 5] - __popc(m & ((1u << (d & 31)) - 1u));
                if (rank < kQaListCap) listed[rank] = (unsigned short)d;
            }
        }
        __syncthreads();
    }
    const int L = two_pass ? n_listed : 0;
    const bool use_list = two_pass && L <= kQaListCap;   // else: listed dwords are done in pass 1
    // One trip to memory per workgroup for what the listed elements need besides their values;
    // pass 2 is then a single load per element instead of a chain of four.
    const bool use_meta = use_list && L <= meta_cap;
    if (use_meta) {
        for (int idx = threadIdx.x; idx < 4 * L; idx += kThreads) {
            const int k = 4 * (int)listed[idx >> 2] + (idx & 3);
            int col = -1, dep = 0;
            uint32_t path = 0u;
            if (k < Ke) {
                const int j = k / g, t = k - j * g;
                int src = chan_src[j];
                src = src < 0 ? 0 : (src >= C ? C - 1 : src);
                col = src * g + t;
                dep = chan_depth[j] < 31 ? chan_depth[j] : 31;
                path = chan_path[j];
            }
            meta_col[idx] = col;
            meta_path[idx] = path;
            meta_dep[idx] = (unsigned char)(dep < 0 ? 0 : dep);
        }
        __syncthreads();
    }

    // the grid: threshold *thr, step T / qmax; written out as {T, step} when the caller wants it
    // (scale_out is then another buffer than thr)
    const float T = thr[0];
    const float step = T / qmax;
    const float half_step = step * 0.5f;
    if (scale_out != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        scale_out[0] = T;
        scale_out[1] = step;
    }
    float inv = 0.0f;
    if (T > 0.0f) inv = __builtin_fminf(__fdiv_rn(qmax, T), 3.402823466e+38f);

    const Index total = (Index)N * (Index)D;
    const Index stride = (Index)gridDim.x * kThreads;
    auto locate = [&](Index o, int64_t& n, int& d) {
        if (sizeof(Index) == 4) {   // division by D: multiply by floor(2^32 / D), one correction
            unsigned q = __umulhi((unsigned)o, magic);
            unsigned r = (unsigned)o - q * (unsigned)D;
            if (r >= (unsigned)D) { ++q; r -= (unsigned)D; }
            n = q;
            d = (int)r;
        } else {
            n = (int64_t)(o / (Index)D);
            d = (int)(o - (Index)n * (Index)D);
        }
    };
    if (!use_list) {
        // every dword by the element-by-element member (fp32 output wanted, or a row too long for
        // the mask or the list)
        for (Index o = (Index)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
            int64_t n;
            int d;
            locate(o, n, d);
            const unsigned packed = qa_dword_generic(W, ldw, n, d, C, g, Ke, chan_src, chan_depth,
                                                     chan_path, half_step, inv, qmax, W_out, ldo);
            if (Wq) reinterpret_cast<unsigned*>(Wq)[o] = packed;
        }
        return;
    }
    // Pass 1.  One item per trip; the next item's 16-byte load is requested before this one is
    // rounded.  The loop holds no other memory access than that load and the item's store, and
    // the load is unconditional (a listed or padding dword loads its row's first 16 bytes and
    // drops them): with a second path that loads inside the loop, or a load under a divergent
    // condition, the compiler waits for ALL outstanding accesses before every use, the request
    // just made included, and the pass ran at half its rate.
    auto fetch = [&](Index o, f32x4& v, int& d, bool& plain) {
        const Index oc = o < total ? o : total - 1;
        int64_t n;
        locate(oc, n, d);
        plain = (plain_mask[d >> 5] >> (d & 31)) & 1u;
        v = *reinterpret_cast<const f32x4u*>(W + n * ldw + (plain ? 4 * d : 0));
    };
    // The listed dwords and the rest of the output are disjoint, so the two passes need no order
    // between them: with the metadata in LDS the first n2 workgroups (the first dispatched, about
    // one per CU) do pass 2 only and all others pass 1 only, at the same time, and the gathers'
    // trips to memory hide behind the stream instead of following it.
    const int n2 = (use_meta && L > 0 && (int)gridDim.x >= 4 * side_wgs) ? side_wgs : 0;
    if ((int)blockIdx.x >= n2) {
        const Index stride1 = (Index)((int)gridDim.x - n2) * kThreads;
        Index o = (Index)((int)blockIdx.x - n2) * kThreads + threadIdx.x;
        f32x4 cur, nxt;
        int d, nd;
        bool plain, nplain;
        fetch(o, cur, d, plain);
        for (; o < total; o += stride1) {
            fetch(o + stride1, nxt, nd, nplain);
            unsigned packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float p = cur[e] * inv;
                p = __builtin_amdgcn_fmed3f(p, -qmax, qmax);
                packed |= ((unsigned)(int)floorf(p + 0.5f) & 0xFFu) << (8 * e);
            }
            // listed dwords are left to pass 2; the zero padding past the expanded columns is written here
            if (plain || d >= Dk) reinterpret_cast<unsigned*>(Wq)[o] = plain ? packed : 0u;
            cur = nxt;
            d = nd;
            plain = nplain;
        }
    }
    if (L == 0 || (n2 > 0 && (int)blockIdx.x >= n2)) return;
    // pass 2: item t = (row t / L, listed dword t % L), dense
    const int64_t items = N * (int64_t)L;
    const int64_t stride2 = (int64_t)(n2 > 0 ? n2 : (int)gridDim.x) * kThreads;
    if (!use_meta) {
        for (int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x; t < items; t += stride2) {
            const int64_t n = t / L;
            const int d = listed[(int)(t - n * L)];
            reinterpret_cast<unsigned*>(Wq)[n * D + d] =
                qa_dword_generic(W, ldw, n, d, C, g, Ke, chan_src, chan_depth, chan_path, half_step, inv,
                                 qmax, nullptr, 0);
        }
        return;
    }
    constexpr int UN = 4;   // items per trip: the sixteen gathers are all requested before any is used
    for (int64_t t0 = (int64_t)blockIdx.x * kThreads + threadIdx.x; t0 < items; t0 += UN * stride2) {
        int64_t n[UN];
        int i[UN];
        float x[UN][4];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int64_t t = t0 + u * stride2 < items ? t0 + u * stride2 : items - 1;   // surplus: repeats the last item
            n[u] = t / L;
            i[u] = (int)(t - n[u] * L);
            const float* wrow = W + n[u] * ldw;
            const i32x4 cols = *reinterpret_cast<const i32x4*>(&meta_col[4 * i[u]]);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[u][e] = wrow[cols[e] < 0 ? 0 : cols[e]];
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            if (t0 + u * stride2 >= items) break;
            const i32x4 cols = *reinterpret_cast<const i32x4*>(&meta_col[4 * i[u]]);
            unsigned packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int code = 0;
                if (cols[e] >= 0) {
                    float v = x[u][e];
                    const int depth = meta_dep[4 * i[u] + e];
                    const uint32_t path = meta_path[4 * i[u] + e];
                    for (int b = 0; b < depth; ++b) {
                        const float m = ((path >> b) & 1u) ? v + half_step : v - half_step;
                        v = m * 0.5f;
                    }
                    float p = v * inv;
                    p = __builtin_amdgcn_fmed3f(p, -qmax, qmax);
                    code = (int)floorf(p + 0.5f);
                }
                packed |= ((unsigned)code & 0xFFu) << (8 * e);
            }
            reinterpret_cast<unsigned*>(Wq)[n[u] * D + listed[i[u]]] = packed;
        }
    }
}

hipError_t launch_qa_paths(const int32_t* split_src, int C, int s, uint32_t* chan_path,
                           hipStream_t stream) {
    size_t lds = (size_t)(C + s) * 5 + 16;   // C + s <= kMaxExpanded: at most 40 KB
    const int staged = lds + (size_t)s * 4 <= 60 * 1024;
    if (staged) lds += (size_t)s * 4;
    qa_paths_kernel<<<1, kThreads, lds, stream>>>(split_src, C, s, chan_path, staged);
    return hipGetLastError();
}

hipError_t launch_expand_quantize_qa(const float* W, int64_t ldw, int64_t N, int C, int g, int s,
                                     const int32_t* chan_src, const int32_t* chan_depth,
                                     const uint32_t* chan_path, const float* thr, float* scale_out,
                                     float qmax, float* W_out, int64_t ldo, int8_t* Wq, int64_t ldq,
                                     hipStream_t stream) {
    // without codes the fp32 tensor is still walked in groups of four columns
    const int64_t Ke = (int64_t)(C + s) * g;
    const int D = (int)(Wq ? ldq / 4 : ceil_div(Ke, 4));
    const int64_t total = N * D;
    int64_t grid = ceil_div(total, kThreads);
    if (grid > 2048) grid = 2048;   // 8 workgroups per CU, each walking the range with a grid stride
    const unsigned magic = (unsigned)((((uint64_t)1) << 32) / (uint64_t)D);   // D >= 1
    // LDS for the listed dwords' metadata: at most s channels are split (each touches at most
    // (g + 3) / 4 + 1 dwords) and s * g columns are appended; a row with more listed dwords than
    // this allows takes the look-ups in global memory
    int64_t meta_cap = (int64_t)s * ((g + 3) / 4 + 2) + ((int64_t)s * g + 3) / 4 + 4;
    if (meta_cap > kQaMetaCap) meta_cap = kQaMetaCap;
    if (Wq == nullptr || W_out != nullptr) meta_cap = 0;
    const unsigned lds = (unsigned)(meta_cap * 36);   // 16 + 16 + 4 bytes per dword
    if (D >= 2 && total + 4 * grid * kThreads < ((int64_t)1 << 32))   // the loop looks 4 strides ahead
        expand_quantize_qa_kernel<uint32_t><<<dim3((unsigned)grid), kThreads, lds, stream>>>(
            W, ldw, N, C, g, s, chan_src, chan_depth, chan_path, thr, scale_out, qmax, W_out, ldo, Wq, D,
            magic, (int)meta_cap, 256);
    else
        expand_quantize_qa_kernel<uint64_t><<<dim3((unsigned)grid), kThreads, lds, stream>>>(
            W, ldw, N, C, g, s, chan_src, chan_depth, chan_path, thr, scale_out, qmax, W_out, ldo, Wq, D,
            magic, (int)meta_cap, 256);
    return hipGetLastError();
}

// Weight side of Eq. 4 on codes: the copies of a duplicated channel are un-scaled, so their
// codes are byte copies of the source channel's codes, and the first C*g columns never change.
// Per batch only the appended columns (and the padding) are rewritten.
__global__ __launch_bounds__(kThreads) void dup_code_columns_kernel(int8_t* __restrict__ Wq, int64_t ldq,
                                                                    int64_t N, int C, int g, int s,
                                                                    const int32_t* __restrict__ chan_src) {
    const int tail = (int)(ldq - (int64_t)C * g);                // appended + padding columns per row
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o >= N * tail) return;
    const int64_t n = o / tail;
    const int k = C * g + (int)(o - n * tail);
    int8_t code = 0;
    if (k < (C + s) * g) {
        const int j = k / g, t = k - j * g;
        int src = chan_src[j];
        src = src < 0 ? 0 : (src >= C ? C - 1 : src);
        code = Wq[n * ldq + (int64_t)src * g + t];
    }
    Wq[n * ldq + k] = code;
}

hipError_t launch_dup_code_columns(int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int s,
                                   const int32_t* chan_src, hipStream_t stream) {
    const int64_t total = N * (ldq - (int64_t)C * g);
    if (total <= 0) return hipSuccess;
    if (ceil_div(total, kThreads) > 0x7FFFFFFF) return hipErrorInvalidValue;   // one lane per byte: grid.x
    dup_code_columns_kernel<<<dim3((unsigned)ceil_div(total, kThreads)), kThreads, 0, stream>>>(
        Wq, ldq, N, C, g, s, chan_src);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// The expanded layer of Eq. 3 run without expanding it.  A duplicated activation channel
// multiplies each of its weight copies by the same activation code, so the accumulator of the
// expanded layer equals that of an un-expanded layer whose weight code for channel c is the sum
// of the codes of c's copies.  int8 has room for that sum whenever copies * qmax <= 127, i.e.
// for every weight width below 8 bits at the split counts the paper uses.  Off-line, small.
// ---------------------------------------------------------------------------------------------
__global__ void fold_init_kernel(int32_t* max_abs) { *max_abs = 0; }

__global__ __launch_bounds__(kThreads) void fold_weights_kernel(
    const int8_t* __restrict__ Wq, int64_t ldq, int64_t N, int C, int g, int s,
    const int32_t* __restrict__ chan_src, int8_t* __restrict__ Wf, int64_t ldf,
    int32_t* __restrict__ max_abs) {
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    int worst = 0;
    if (o < N * ldf) {
        const int64_t n = o / ldf;
        const int k = (int)(o - n * ldf);
        int sum = 0;
        if (k < C * g) {
            const int c = k / g, t = k - c * g;
            sum = Wq[n * ldq + k];                       // the channel's own slot
            for (int j = C; j < C + s; ++j) {
                int src = chan_src[j];
                src = src < 0 ? 0 : (src >= C ? C - 1 : src);
                if (src == c) sum += Wq[n * ldq + (int64_t)j * g + t];
            }
        }
        worst = sum < 0 ? -sum : sum;
        Wf[o] = (int8_t)(sum > 127 ? 127 : (sum < -127 ? -127 : sum));
    }
    const unsigned w = wave_umax32((unsigned)worst);
    if ((threadIdx.x & 63) == 0 && w != 0u) atomicMax(max_abs, (int)w);
}

hipError_t launch_fold_weights(const int8_t* Wq, int64_t ldq, int64_t N, int C, int g, int s,
                               const int32_t* chan_src, int8_t* Wf, int64_t ldf, int32_t* max_abs,
                               hipStream_t stream) {
    if (ceil_div(N * ldf, kThreads) > 0x7FFFFFFF) return hipErrorInvalidValue;   // one lane per byte: grid.x
    fold_init_kernel<<<1, 1, 0, stream>>>(max_abs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    fold_weights_kernel<<<dim3((unsigned)ceil_div(N * ldf, kThreads)), kThreads, 0, stream>>>(
        Wq, ldq, N, C, g, s, chan_src, Wf, ldf, max_abs);
    return hipGetLastError();
}

}  // namespace ocs
