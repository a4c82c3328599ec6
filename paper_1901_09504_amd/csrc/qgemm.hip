// The expanded layer (Eq. 2 over the expanded channel set) on int8 codes: an NT GEMM
// acc[i,n] = sum_k Xq[i,k] * Wq[n,k] on the matrix cores (v_mfma_i32_32x32x32_i8, int32
// accumulation, exact), with the trailing scale factors of Eq. 1 applied in the epilogue.
//
// Both operands are K-contiguous, so a lane's MFMA operand is 16 consecutive bytes of one
// row.  A workgroup computes a BM x BN tile; per K-step of 64 or 128 bytes the BM + BN row
// segments go from global memory straight into LDS (no staging registers), into a ring of
// buffers (long K) or all at once (short K).  LDS rows are BK bytes = 16-byte chunks whose
// index is XOR-swizzled with the row so that the 16-byte fragment reads of consecutive rows fall
// in different banks.  K is padded with zero codes to a multiple of 64 by the producers, so the
// K loop has no tail; zeros add nothing to an integer sum.
#include <atomic>

#include "ocs_internal.h"

namespace ocs {

// LDS rows are BK bytes = BK/16 chunks of 16 bytes.  The chunk index is XOR-ed with a function
// of the row chosen so that the 16-byte reads of 8 (and of 16) consecutive rows at one K offset
// land in distinct bank groups.
template <int BK>
__device__ __forceinline__ int swz(int row, int chunk) {
    if (BK == 64) return chunk ^ (((row >> 2) & 3) ^ (row & 2));
    return chunk ^ (((row >> 1) & 7) ^ ((row & 1) << 2));
}

// index clamped into [0, n): index arrays and edge rows never send a load out of bounds
__device__ __forceinline__ int col_clamp(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber them so
// that consecutive tile ids (which share an X row panel) run on the same XCD.
__device__ __forceinline__ unsigned xcd_remap(unsigned w, unsigned total) {
    const unsigned q = total / 8, r = total % 8;
    const unsigned xcd = w % 8, local = w / 8;
    return xcd * q + (xcd < r ? xcd : r) + local;
}

// ---------------------------------------------------------------------------------------------
// The operands move global -> LDS directly (global_load_lds_dwordx4): no staging registers and no
// LDS write instructions, which on this chip cost as much LDS time as the fragment reads (the LDS
// takes ~73 B/clk of writes against ~190 B/clk of 16-byte reads).
// One such instruction fills 1 KB of LDS, lane l at byte 16*l of the wave's block (the block
// base travels in M0 and is wave-uniform), so the XOR swizzle is applied on the global side:
// the lane that fills chunk slot c of row r fetches chunk c ^ f(r) of that row.  NBUF LDS
// buffers form the prefetch ring; a wave waits for its own loads of the next step with vmcnt
// (loads return in order), and the step's barrier then makes every wave's part visible.
// ---------------------------------------------------------------------------------------------
template <int N_>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N_ >= 0 && N_ < 64, "vmcnt is a 6-bit counter");
    // s_waitcnt simm16: vmcnt[3:0], expcnt[6:4], lgkmcnt[11:8], vmcnt[5:4] in bits 15:14
    __builtin_amdgcn_s_waitcnt((N_ & 15) | (7 << 4) | (15 << 8) | ((N_ >> 4) << 14));
}

__device__ __forceinline__ unsigned out_code(int a, float scale, int relu, float inv, float qmax) {
    float y = (float)a * scale;
    if (relu) y = y > 0.0f ? y : 0.0f;
    float p = y * inv;
    p = __builtin_amdgcn_fmed3f(p, -qmax, qmax);
    return __float_as_uint(p + 12582912.0f) & 0xFFu;   // round half to even; low byte = code
}

// Copies the next layer wants of this workgroup's output columns: entries (j << 8 | column
// inside the workgroup's BN columns) for every appended column N + j whose source lies in
// [col0, col0 + BN).  Built once per workgroup (a handful of entries: a few percent of BN).
constexpr int kDupCap = 512;
template <int NT>
__device__ __forceinline__ void build_dup_list(const Requant& rq, int N, int col0, int BN_, int* list,
                                               int* count) {
    if (rq.Yq == nullptr || rq.s_next <= 0) return;   // uniform over the grid
    if (threadIdx.x == 0) *count = 0;
    __syncthreads();
    for (int t = threadIdx.x; t < rq.s_next; t += NT) {
        int src = rq.chan_src[N + t];
        src = src < 0 ? 0 : (src >= N ? N - 1 : src);
        const int local = src - col0;
        if (local >= 0 && local < BN_) {
            const int k = atomicAdd(count, 1);
            if (k < kDupCap) list[k] = (t << 8) | local;
        }
    }
    __syncthreads();
}

// ROWS x WN accumulators of one wave, staged row-major in its piece of LDS, go out to memory.
// rbase / cbase: global row and column of the staged block's corner; wcol: its first column
// inside the workgroup's tile.  fp32 (and the optional int32 dump): lane = (row, four
// consecutive columns), 16-byte stores.  Codes: lane = (row, sixteen consecutive columns),
// again 16-byte stores.
template <int ROWS, int WN>
__device__ __forceinline__ void emit_staged_rows(const int32_t* stage, int lane, int rbase, int cbase,
                                                 int wcol, int M, int N, float scale,
                                                 float* __restrict__ Y, int64_t ldy,
                                                 int32_t* __restrict__ acc_out, int64_t ldacc,
                                                 bool vec_y, bool vec_a, const Requant& rq, float inv,
                                                 const int* dup_list, int dup_n, bool pad_writer) {
    constexpr int LPR = WN / 4;            // lanes per row (8, 16 or 32)
    constexpr int SLOTS = ROWS * LPR;      // 16-byte reads of the block
    static_assert(SLOTS % 64 == 0, "whole waves of slots");
    if (rq.Yq == nullptr || acc_out != nullptr) {
#pragma unroll
        for (int it = 0; it < SLOTS / 64; ++it) {
            const int idx = it * 64 + lane;
            const int rr = idx / LPR, cc = (idx % LPR) * 4;
            const i32x4 a = *reinterpret_cast<const i32x4*>(&stage[rr * WN + cc]);
            const int r = rbase + rr, c = cbase + cc;
            if (r >= M || c >= N) continue;
            if (rq.Yq == nullptr) {
                float* yp = Y + (int64_t)r * ldy + c;
                if (vec_y && c + 3 < N) {
                    f32x4 y;
#pragma unroll
                    for (int e = 0; e < 4; ++e) y[e] = (float)a[e] * scale;
                    __builtin_nontemporal_store(y, reinterpret_cast<f32x4*>(yp));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < N) yp[e] = (float)a[e] * scale;
                }
            }
            if (acc_out) {
                int32_t* ap = acc_out + (int64_t)r * ldacc + c;
                if (vec_a && c + 3 < N) {
                    *reinterpret_cast<i32x4*>(ap) = a;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c + e < N) ap[e] = a[e];
                }
            }
        }
    }
    if (rq.Yq == nullptr) return;

    constexpr int LPR16 = WN / 16;         // lanes per row, sixteen columns each (2, 4 or 8)
    constexpr int SLOTS16 = ROWS * LPR16;
#pragma unroll
    for (int it = 0; it < (SLOTS16 + 63) / 64; ++it) {
        const int idx = it * 64 + lane;
        if (idx >= SLOTS16) break;
        const int rr = idx / LPR16, cc = (idx % LPR16) * 16;
        const int r = rbase + rr, c = cbase + cc;
        unsigned w[4];
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const i32x4 a = *reinterpret_cast<const i32x4*>(&stage[rr * WN + cc + 4 * g4]);
            w[g4] = out_code(a[0], scale, rq.relu, inv, rq.qmax) |
                    (out_code(a[1], scale, rq.relu, inv, rq.qmax) << 8) |
                    (out_code(a[2], scale, rq.relu, inv, rq.qmax) << 16) |
                    (out_code(a[3], scale, rq.relu, inv, rq.qmax) << 24);
        }
        if (r >= M || c >= N) continue;
        int8_t* qp = rq.Yq + (int64_t)r * rq.ldyq + c;      // 16-byte aligned: ldyq % 16 == 0, c % 16 == 0
        if (c + 15 < N) {
            i32x4 v;
            v[0] = (int)w[0]; v[1] = (int)w[1]; v[2] = (int)w[2]; v[3] = (int)w[3];
            *reinterpret_cast<i32x4*>(qp) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (c + e < N) qp[e] = (int8_t)((w[e >> 2] >> (8 * (e & 3))) & 0xFFu);
        }
    }
    // copies for the channels the next layer splits: the wave that holds the source column
    // writes appended column N + j, one lane per staged row
    if (dup_n > 0 && lane < ROWS) {
        const int r = rbase + lane;
        for (int k = 0; k < dup_n; ++k) {
            const int e = dup_list[k];
            const int local = (e & 0xFF) - wcol;
            if (local >= 0 && local < WN && r < M)
                rq.Yq[(int64_t)r * rq.ldyq + N + (e >> 8)] =
                    (int8_t)out_code(stage[lane * WN + local], scale, rq.relu, inv, rq.qmax);
        }
    }
    // the pad columns of the code tensor (past the last copy) are zero codes: written by one wave
    // of the last tile column, one lane per staged row
    if (pad_writer && lane < ROWS) {
        const int r = rbase + lane;
        if (r < M)
            for (int64_t c = (int64_t)N + rq.s_next; c < rq.ldyq; ++c) rq.Yq[(int64_t)r * rq.ldyq + c] = 0;
    }
}

__device__ __forceinline__ float requant_inv(const Requant& rq, bool writer) {
    if (rq.Yq == nullptr) return 0.0f;
    const float T = *rq.thr;
    if (writer && rq.scale_out != nullptr) {
        rq.scale_out[0] = T;
        rq.scale_out[1] = T / rq.qmax;
    }
    if (!(T > 0.0f)) return 0.0f;
    return __builtin_fminf(__fdiv_rn(rq.qmax, T), 3.402823466e+38f);
}

// Geometry of a convolution whose lowering to the GEMM is done by the A-operand loader itself
// (CONV variant below): the un-lowered activation codes Aq [B, H, W, ldc] (ldc bytes per pixel,
// a multiple of 16: the expanded channels first, zero padding after), kernel kh x kw, output
// Ho x Wo.  K is walked tap by tap in 16-byte chunks: chunk G of a row is chunk G % cpp of tap
// G / cpp, cpp = ldc / 16 chunks per pixel, so a lane's 16 bytes are 16 consecutive channels of
// one input pixel.  Taps that fall outside the image, and the chunks that pad K up to a whole
// K-step after the last tap, read a row of zeros instead.
struct ConvGeom {
    const int8_t* zero;   // at least BK bytes of zeros
    int H, W, kh, kw, cpp, stride, pad, Ho, Wo;
    int64_t ldc;
};

// K split across workgroups: `parts` workgroups share one output tile, each walks its own slice of
// the K-steps, stores its int32 accumulators in partials[tile][part] (in the register layout, so
// that the stores and the loads are whole 1 KB wave accesses) and signs in at counters[tile]; the
// one that signs in last adds the others' accumulators to its own (integer sums: any order gives
// the same bits) and runs the epilogue.  Nobody waits for anybody.  A counter wraps back to zero
// with the last arrival (atomicInc), so the counters only have to be zero once.
struct SplitK {
    int32_t* partials = nullptr;   // [tiles][parts][BM * BN]
    unsigned* counters = nullptr;  // [tiles], zero between launches
    int parts = 1;
};

// Sixteen zero codes: what a row "holds" past its pitch.  With a short K the rows of the operands
// need not fill their last K-step (a 68-byte row in an 80-byte pitch, walked as 128 bytes): the
// 16-byte pieces that lie past the pitch are fetched from here instead of from the next row.
__device__ __align__(16) int8_t zero_chunk[16] = {};   // (not declared const: it must stay in the global address space, like the rows it stands in for)

// MASK: the pitches may end inside the last K-step (see zero_chunk); every request then checks
// its piece against the pitch.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NBUF, bool CONV = false, bool SPLIT = false,
          bool MASK = false>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void qgemm_dma_kernel(
    const int8_t* __restrict__ Xq, int64_t ldx, const int8_t* __restrict__ Wq, int64_t ldw, int M,
    int N, int ksteps_all, const float* __restrict__ scale_x, const float* __restrict__ scale_w,
    int32_t* __restrict__ acc_out, int64_t ldacc, float* __restrict__ Y, int64_t ldy, int tiles_n,
    unsigned total_tiles, ConvGeom cg, Requant rq, SplitK sk) {
    constexpr int NW = WAVES_M * WAVES_N;  // waves (4, 8 or 16)
    constexpr int NT = NW * 64;
    static_assert(NW == 4 || NW == 8 || NW == 16, "4, 8 or 16 waves");
    static_assert(!SPLIT || !CONV, "K split across workgroups: plain GEMM");
    static_assert(!MASK || (!SPLIT && !CONV), "pitch shorter than the K walk: plain GEMM");
    static_assert(BK == 64 || BK == 128, "K-step of 64 or 128 bytes");
    static_assert(NBUF >= 3, "ring of at least three buffers");
    constexpr int CPR = BK / 16;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_LOADS = BM * CPR / NT, B_LOADS = BN * CPR / NT;  // per wave & step
    constexpr int LPS = A_LOADS + B_LOADS;
    static_assert(A_LOADS >= 1 && B_LOADS >= 1, "tile too small");
    static_assert((NBUF - 2) * LPS < 64, "prefetch ring exceeds the vmcnt range");
    constexpr int KS = BK / 32;

    // one array: the A ring, then the B ring; the epilogue reuses all of it
    constexpr int RING_BYTES = NBUF * (BM + BN) * BK;
    __shared__ __align__(1024) int8_t lds[RING_BYTES];
    __shared__ int dup_list[kDupCap];
    __shared__ int dup_count;
    int8_t (*lds_a)[BM * BK] = reinterpret_cast<int8_t (*)[BM * BK]>(&lds[0]);
    int8_t (*lds_b)[BN * BK] = reinterpret_cast<int8_t (*)[BN * BK]>(&lds[NBUF * BM * BK]);

    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // SPLIT: the parts of a tile are neighbours in the renumbered order, so they run on one XCD
    // and their partial sums meet in its L2
    const unsigned vwg = xcd_remap(blockIdx.x, SPLIT ? total_tiles * (unsigned)sk.parts : total_tiles);
    const unsigned tile = SPLIT ? vwg / (unsigned)sk.parts : vwg;
    const int part = SPLIT ? (int)(vwg % (unsigned)sk.parts) : 0;
    const int kbeg = SPLIT ? (int)((int64_t)part * ksteps_all / sk.parts) : 0;
    const int ksteps = SPLIT ? (int)((int64_t)(part + 1) * ksteps_all / sk.parts) - kbeg : ksteps_all;
    const int bm = (int)(tile / tiles_n), bn = (int)(tile % tiles_n);
    const int row0 = bm * BM, col0 = bn * BN;

    // Load u of this wave fills LDS block (u*4 + wave): slots p = block*64 + lane, row p / CPR,
    // chunk slot p % CPR, which receives global chunk slot ^ f(row).
    const int8_t* a_src[A_LOADS];
    const int8_t* b_src[B_LOADS];
    // CONV: output pixel of each row this lane loads (top-left input coordinate of its window,
    // byte offset of that input pixel, which may lie outside the tensor and is then never used),
    // and the tap position (ky, kx, chunk in pixel) of the chunk this lane will request next for
    // that row: chunk kt*CPR + (its swizzled chunk slot) of the row's K extent.
    int a_iy0[CONV ? A_LOADS : 1], a_ix0[CONV ? A_LOADS : 1];
    int a_ky[CONV ? A_LOADS : 1], a_kx[CONV ? A_LOADS : 1], a_cin[CONV ? A_LOADS : 1];
    int a_zoff[CONV ? A_LOADS : 1];
    int a_piece[MASK ? A_LOADS : 1], b_piece[MASK ? B_LOADS : 1];   // MASK: the lane's piece of K-step 0
    const int a_pieces = (int)(ldx / 16), b_pieces = (int)(ldw / 16);
#pragma unroll
    for (int u = 0; u < A_LOADS; ++u) {
        int pslot = (u * NW + wave) * 64 + lane, r = pslot / CPR, c = pslot % CPR;
        if (MASK) a_piece[u] = swz<BK>(r, c);
        int gr = row0 + r;
        gr = gr < M ? gr : M - 1;  // rows past the edge re-read the last row; never stored
        if (CONV) {
            const int per_img = cg.Ho * cg.Wo;
            const int b = gr / per_img, rem = gr - b * per_img;
            const int yo = rem / cg.Wo, xo = rem - yo * cg.Wo;
            a_iy0[u] = yo * cg.stride - cg.pad;
            a_ix0[u] = xo * cg.stride - cg.pad;
            a_src[u] = Xq + (((int64_t)b * cg.H + a_iy0[u]) * cg.W + a_ix0[u]) * cg.ldc;
            a_zoff[u] = swz<BK>(r, c) * 16;
            int cin = swz<BK>(r, c), kx = 0, ky = 0;
            while (cin >= cg.cpp) {
                cin -= cg.cpp;
                if (++kx == cg.kw) { kx = 0; ++ky; }
            }
            a_cin[u] = cin;
            a_kx[u] = kx;
            a_ky[u] = ky;
        } else {
            a_src[u] = Xq + (int64_t)gr * ldx + swz<BK>(r, c) * 16 + (int64_t)kbeg * BK;
        }
    }
    int c_kt = 0;   // CONV: K-step the next request is for (stops at the last one)
#pragma unroll
    for (int u = 0; u < B_LOADS; ++u) {
        int pslot = (u * NW + wave) * 64 + lane, r = pslot / CPR, c = pslot % CPR;
        int gr = col0 + r;
        gr = gr < N ? gr : N - 1;
        b_src[u] = Wq + (int64_t)gr * ldw + swz<BK>(r, c) * 16 + (int64_t)kbeg * BK;
        if (MASK) b_piece[u] = swz<BK>(r, c);
    }

    // The load is issued through inline assembly on purpose: issued through the compiler's
    // builtin, every later LDS read is preceded by a wait for ALL outstanding loads (the
    // compiler cannot tell which LDS bytes a load fills), which would serialise the ring.
    // The waits are placed by hand instead (wait_vmcnt below); the kernel has no other loads
    // in flight until the epilogue, which starts after a wait for zero.
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) int8_t* lptr_t;
    const unsigned lds_a0 = (unsigned)(uintptr_t)(lptr_t)&lds_a[0][0];  // LDS byte addresses
    const unsigned lds_b0 = (unsigned)(uintptr_t)(lptr_t)&lds_b[0][0];
#else
    const unsigned lds_a0 = 0, lds_b0 = 0;
#endif
    auto dma16 = [&](const int8_t* g, unsigned lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
        // the block base is the same for every lane of the wave; M0 wants it in a scalar register
        const unsigned m0 = __builtin_amdgcn_readfirstlane(lds_addr);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :
                     : "v"(g), "s"(m0)
                     : "memory");
#else
        (void)g;
        (void)lds_addr;
#endif
    };
    auto fetch = [&](int kt, int buf) {   // K index clamped: surplus steps refetch the last one
        const int kl = kt < ksteps ? kt : ksteps - 1;
        const int64_t koff = (int64_t)kl * BK;
        if (CONV) {
            // requests arrive in K order, so each lane keeps the tap position of its chunk
            // incrementally; it stops at the last step, which surplus requests repeat
            const bool advance = c_kt + 1 < ksteps;
#pragma unroll
            for (int u = 0; u < A_LOADS; ++u) {
                const int iy = a_iy0[u] + a_ky[u], ix = a_ix0[u] + a_kx[u];
                const bool inside = a_ky[u] < cg.kh && (unsigned)iy < (unsigned)cg.H &&
                                    (unsigned)ix < (unsigned)cg.W;
                const int8_t* src =
                    inside ? a_src[u] + ((int64_t)a_ky[u] * cg.W + a_kx[u]) * cg.ldc + a_cin[u] * 16
                           : cg.zero + a_zoff[u];
                dma16(src, lds_a0 + buf * (BM * BK) + (u * NW + wave) * 1024);
                if (advance) {
                    int cin = a_cin[u] + CPR, kx = a_kx[u], ky = a_ky[u];
                    while (cin >= cg.cpp) {
                        cin -= cg.cpp;
                        if (++kx == cg.kw) { kx = 0; ++ky; }
                    }
                    a_cin[u] = cin;
                    a_kx[u] = kx;
                    a_ky[u] = ky;
                }
            }
            if (advance) ++c_kt;
        } else {
#pragma unroll
            for (int u = 0; u < A_LOADS; ++u)
                dma16(!MASK || kl * CPR + a_piece[u] < a_pieces ? a_src[u] + koff : zero_chunk,
                      lds_a0 + buf * (BM * BK) + (u * NW + wave) * 1024);
        }
#pragma unroll
        for (int u = 0; u < B_LOADS; ++u)
            dma16(!MASK || kl * CPR + b_piece[u] < b_pieces ? b_src[u] + koff : zero_chunk,
                  lds_b0 + buf * (BN * BK) + (u * NW + wave) * 1024);
    };

    i32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int frag_row = lane & 31, frag_half = lane >> 5;
    i32x4 af[2][TM], bf[2][TN];
    auto read_slice = [&](int buf, int ks, i32x4 (&a)[TM], i32x4 (&b)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int r = wm * WM + i * 32 + frag_row;
            a[i] = *reinterpret_cast<const i32x4*>(
                &lds_a[buf][r * BK + swz<BK>(r, ks * 2 + frag_half) * 16]);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int r = wn * WN + j * 32 + frag_row;
            b[j] = *reinterpret_cast<const i32x4*>(
                &lds_b[buf][r * BK + swz<BK>(r, ks * 2 + frag_half) * 16]);
        }
    };
    auto multiply = [&](i32x4 (&a)[TM], i32x4 (&b)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    };

    // Step kt multiplies out of buffer kt % NBUF.  At its start it requests step kt+NBUF-1 into
    // the buffer step kt-1 used (every wave finished reading it before the previous barrier).
    // Before its last slice it waits until only the loads of steps kt+2.. are outstanding,
    // takes the barrier, and requests slice 0 of step kt+1.
    auto step = [&](int buf, int kt) {
        fetch(kt + NBUF - 1, (buf + NBUF - 1) % NBUF);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) {
                read_slice(buf, ks + 1, af[(ks + 1) & 1], bf[(ks + 1) & 1]);
            } else {
                wait_vmcnt<(NBUF - 2) * LPS>();
                __syncthreads();
                read_slice((buf + 1) % NBUF, 0, af[0], bf[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
            multiply(af[ks & 1], bf[ks & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

#pragma unroll
    for (int p = 0; p < NBUF - 1; ++p) fetch(p, p);
    build_dup_list<NT>(rq, N, col0, BN, dup_list, &dup_count);   // behind the first requests
    wait_vmcnt<(NBUF - 2) * LPS>();
    __syncthreads();
    read_slice(0, 0, af[0], bf[0]);

    const int gsteps = ksteps;
    int kt0 = 0;
    for (; kt0 + NBUF <= gsteps; kt0 += NBUF) {
#pragma unroll
        for (int p = 0; p < NBUF; ++p) step(p, kt0 + p);
    }
#pragma unroll
    for (int p = 0; p < NBUF; ++p)
        if (kt0 + p < gsteps) step(p, kt0 + p);
    wait_vmcnt<0>();  // surplus (clamped) loads must land before the ring is reused below
    __syncthreads();  // every wave has read its last fragments: the rings are free

    if constexpr (SPLIT) {
        // The partial sums cross between workgroups that may sit on different XCDs, each with an
        // L2 of its own.  They are stored and loaded as device-coherent accesses (the sc1 bit:
        // written through to, and read from, the memory side of the L2s), which needs no cache
        // maintenance: a device-scope fence instead writes back and invalidates a whole L2 per
        // workgroup (measured: 120 us instead of 42 on the 512-channel 3x3 layer).  Order: stores,
        // wait until they are acknowledged, barrier, one arrival per workgroup.
        __shared__ unsigned arrival;
        constexpr int WAVE_VEC = TM * TN * 4 * 64;   // 16-byte groups of one wave's accumulators
        i32x4* mine = reinterpret_cast<i32x4*>(sk.partials + ((size_t)tile * sk.parts + part) * (size_t)(BM * BN)) +
                      (size_t)wave * WAVE_VEC + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int vg = 0; vg < 4; ++vg) {
                    i32x4 v;
                    v[0] = acc[i][j][4 * vg]; v[1] = acc[i][j][4 * vg + 1];
                    v[2] = acc[i][j][4 * vg + 2]; v[3] = acc[i][j][4 * vg + 3];
                    i32x4* dst = mine + ((i * TN + j) * 4 + vg) * 64;
#if defined(__HIP_DEVICE_COMPILE__)
                    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst), "v"(v) : "memory");
#else
                    *dst = v;
#endif
                }
        wait_vmcnt<0>();          // every store of this wave has been acknowledged
        __syncthreads();
        if (threadIdx.x == 0) arrival = atomicInc(sk.counters + tile, (unsigned)sk.parts - 1u);
        __syncthreads();
        if (arrival != (unsigned)sk.parts - 1u) return;   // not the last one: done (no barrier follows)
        for (int q = 0; q < sk.parts; ++q) {
            if (q == part) continue;
            const i32x4* theirs = reinterpret_cast<const i32x4*>(
                                      sk.partials + ((size_t)tile * sk.parts + q) * (size_t)(BM * BN)) +
                                  (size_t)wave * WAVE_VEC + lane;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    i32x4 v0, v1, v2, v3;
                    const i32x4* src = theirs + ((i * TN + j) * 4) * 64;
#if defined(__HIP_DEVICE_COMPILE__)
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v0) : "v"(src) : "memory");
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v1) : "v"(src + 64) : "memory");
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v2) : "v"(src + 128) : "memory");
                    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v3) : "v"(src + 192) : "memory");
                    // the sums below must not be scheduled ahead of the wait: they take their
                    // operands from it
                    asm volatile("s_waitcnt vmcnt(0)" : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3) : : "memory");
#else
                    v0 = src[0]; v1 = src[64]; v2 = src[128]; v3 = src[192];
#endif
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[i][j][e] += v0[e];
                        acc[i][j][4 + e] += v1[e];
                        acc[i][j][8 + e] += v2[e];
                        acc[i][j][12 + e] += v3[e];
                    }
                }
        }
    }

    // Epilogue.  An accumulator block leaves the MFMA with lane l holding ONE column and 16
    // rows, which as stores would be 4 bytes per lane (measured: a CU retires such stores at
    // ~16 B/clk, which made the output-bound shapes run at half the HBM write rate).  Each wave
    // therefore turns its accumulators through a private piece of the free ring, 32 rows at a
    // time, and reads them back with each lane holding four consecutive columns of one row:
    // 16-byte stores, whole 128-byte lines per row.  Only this wave touches its piece and a
    // wave's LDS accesses execute in issue order, so no barrier is needed.
    constexpr int WAVE_STAGE = RING_BYTES / NW;          // bytes of LDS per wave
    static_assert(WAVE_STAGE >= 32 * WN * 4, "ring too small to stage 32 rows of a wave's tile");
    static_assert(WAVE_STAGE % 16 == 0, "staging area must keep 16-byte alignment");
    int32_t* stage = reinterpret_cast<int32_t*>(&lds[wave * WAVE_STAGE]);
    const float scale = scale_x[1] * scale_w[1];
    const float inv = requant_inv(rq, (SPLIT ? tile == 0 : blockIdx.x == 0) && threadIdx.x == 0);
    const int dup_n = (rq.Yq != nullptr && rq.s_next > 0) ? (dup_count < kDupCap ? dup_count : kDupCap) : 0;
    const bool vec_y = (reinterpret_cast<uintptr_t>(Y) % 16 == 0) && (ldy % 4 == 0);
    const bool vec_a = acc_out != nullptr && (reinterpret_cast<uintptr_t>(acc_out) % 16 == 0) &&
                       (ldacc % 4 == 0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                stage[((v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * WN + j * 32 + (lane & 31)] =
                    acc[i][j][v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        emit_staged_rows<32, WN>(stage, lane, row0 + wm * WM + i * 32, col0 + wn * WN, wn * WN, M, N,
                                 scale, Y, ldy, acc_out, ldacc, vec_y, vec_a, rq, inv, dup_list, dup_n,
                                 rq.Yq != nullptr && bn == tiles_n - 1 && wn == 0);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // the reads are issued before the next block's writes
    }
}

// ---------------------------------------------------------------------------------------------
// Short-K variant: the whole K extent of the tile's operands (ksteps steps of 64 bytes) is
// requested into LDS up front, with no ring and no surplus requests, multiplied after ONE wait
// and barrier, and the workgroup keeps no more LDS than that (dynamic size).  For the layers
// with a few hundred input channels the GEMM is a stream of 4*N output bytes per row: what
// matters there is how many workgroups a CU holds, so that one's request latency hides behind
// the others' stores.  Per K-step the LDS holds BM rows of A, then BN rows of B, 64 bytes each,
// chunk-swizzled like the ring kernel's.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_dma16(const int8_t* g, unsigned lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
    const unsigned m0 = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(g), "s"(m0)
                 : "memory");
#else
    (void)g;
    (void)lds_addr;
#endif
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void qgemm_wholek_kernel(
    const int8_t* __restrict__ Xq, int64_t ldx, const int8_t* __restrict__ Wq, int64_t ldw, int M,
    int N, int ksteps, const float* __restrict__ scale_x, const float* __restrict__ scale_w,
    int32_t* __restrict__ acc_out, int64_t ldacc, float* __restrict__ Y, int64_t ldy, int tiles_n,
    unsigned total_tiles, int dup_off, Requant rq) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS = BM + BN;          // LDS rows per K-step
    constexpr int STEP_BYTES = ROWS * 64;
    constexpr int BLOCKS = ROWS / 16;      // 1 KB pieces per K-step, 16 rows each
    static_assert(BM % 16 == 0 && BN % 16 == 0, "a 1 KB piece must not straddle the operands");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && TM >= 1 && TN >= 1, "wave tile of 32x32 blocks");

    // No static LDS here: at 320 bytes of K a 128x128 tile's operands are exactly half of a
    // CU's LDS, and a few bytes more would halve the workgroups a CU holds.  The table of the
    // next layer's copies follows the operands, and only when the epilogue needs it.
    extern __shared__ __align__(1024) int8_t dlds[];
    int* dup_list = reinterpret_cast<int*>(&dlds[dup_off]);   // used only when dup_off > 0
    int* dup_count = dup_list + kDupCap;
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) int8_t* lptr_t;
    const unsigned lds0 = (unsigned)(uintptr_t)(lptr_t)&dlds[0];
#else
    const unsigned lds0 = 0;
#endif

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const unsigned tile = xcd_remap(blockIdx.x, total_tiles);
    const int bm = (int)(tile / tiles_n), bn = (int)(tile % tiles_n);
    const int row0 = bm * BM, col0 = bn * BN;

    // piece b of a K-step: LDS rows 16b .. 16b+15; lane l fills row 16b + l/4, chunk slot l%4
    // (a row's pitch may end inside the last K-step: pieces past it come from zero_chunk)
    for (int b = wave; b < BLOCKS; b += NW) {
        const int r = b * 16 + (lane >> 2), c = lane & 3;
        const int8_t* rowp;
        int piece, pieces;                 // this lane's 16-byte piece of K-step 0; pieces in the pitch
        if (r < BM) {
            int gr = row0 + r;
            gr = gr < M ? gr : M - 1;      // rows past the edge re-read the last row; never stored
            rowp = Xq + (int64_t)gr * ldx;
            piece = swz<64>(r, c);
            pieces = (int)(ldx / 16);
        } else {
            int gr = col0 + (r - BM);
            gr = gr < N ? gr : N - 1;
            rowp = Wq + (int64_t)gr * ldw;
            piece = swz<64>(r - BM, c);
            pieces = (int)(ldw / 16);
        }
        for (int kt = 0; kt < ksteps; ++kt, piece += 4)
            lds_dma16(piece < pieces ? rowp + piece * 16 : zero_chunk, lds0 + kt * STEP_BYTES + b * 1024);
    }

    i32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    if (dup_off > 0) build_dup_list<NW * 64>(rq, N, col0, BN, dup_list, dup_count);   // behind the requests
    wait_vmcnt<0>();
    __syncthreads();

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int kt = 0; kt < ksteps; ++kt) {
        const int8_t* base = &dlds[kt * STEP_BYTES];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            i32x4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int r = wm * WM + i * 32 + frag_row;
                a[i] = *reinterpret_cast<const i32x4*>(
                    &base[r * 64 + swz<64>(r, ks * 2 + frag_half) * 16]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int r = wn * WN + j * 32 + frag_row;
                b[j] = *reinterpret_cast<const i32x4*>(
                    &base[(BM + r) * 64 + swz<64>(r, ks * 2 + frag_half) * 16]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();  // the operands are dead: their LDS becomes the staging area

    // Epilogue as in the ring kernel (each wave turns its accumulators through a private piece
    // of LDS into rows of 16-byte stores), 8 rows at a time to keep the footprint small.
    int32_t* stage = reinterpret_cast<int32_t*>(&dlds[wave * (8 * WN * 4)]);
    const float scale = scale_x[1] * scale_w[1];
    const float inv = requant_inv(rq, blockIdx.x == 0 && tid == 0);
    const int dup_n = dup_off > 0 ? (*dup_count < kDupCap ? *dup_count : kDupCap) : 0;
    const bool vec_y = (reinterpret_cast<uintptr_t>(Y) % 16 == 0) && (ldy % 4 == 0);
    const bool vec_a = acc_out != nullptr && (reinterpret_cast<uintptr_t>(acc_out) % 16 == 0) &&
                       (ldacc % 4 == 0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    stage[((lane >> 5) * 4 + e) * WN + j * 32 + (lane & 31)] = acc[i][j][q * 4 + e];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            emit_staged_rows<8, WN>(stage, lane, row0 + wm * WM + i * 32 + q * 8, col0 + wn * WN, wn * WN,
                                    M, N, scale, Y, ldy, acc_out, ldacc, vec_y, vec_a, rq, inv, dup_list,
                                    dup_n, rq.Yq != nullptr && bn == tiles_n - 1 && wn == 0);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

constexpr int64_t kWholeKMaxLds = 160 * 1024;  // LDS of one CU
constexpr int kMaxDevices = 64;

// Compute units of the current device (looked up once per device; 256 if the query fails).
static int compute_units() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int n = cached[dev].load(std::memory_order_acquire);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev].store(n, std::memory_order_release);
    }
    return n;
}

// ---------------------------------------------------------------------------------------------
// Split + quantize + GEMM in one launch: the A operand is the fp32 activation matrix X [M, C*g]
// itself.  A workgroup takes 128 rows of X and all N <= 256 output columns, walks K in steps of
// 64 source columns, and per step turns its 128 x 64 floats (16-byte loads, two steps ahead, held
// in registers) into codes on the static grid (Eq. 1, the arithmetic of the streaming pass) and
// writes them into LDS in the layout the matrix cores read; the weight codes of the step come
// through registers as well.  The expanded layer's appended channels (the activation side of
// Eq. 3: un-scaled copies) cost no memory traffic at all: the copy of a column is the byte that
// was just written into LDS, so after each step the copies whose sources lie in it are moved,
// byte by byte, into a second LDS area laid out as the K-steps that follow the C*g columns, and
// those steps are multiplied last.  The code tensor Xq never exists in memory: 4 bytes read per
// element of X and 4 written per output, instead of 4 + 1 and 1 + 4 for the two launches.
//
// Per-workgroup set-up: the appended columns e = 0 .. s*g-1 (expanded column C*g + e, source
// column chan_src[C + e/g]*g + e%g) are bucketed by the K-step of their source (counts, prefix,
// fill: three short LDS passes).
// ---------------------------------------------------------------------------------------------
constexpr int kFusedMaxBM = 128;
constexpr int kFusedMaxTail = 2048;    // appended columns s*g
constexpr int kFusedMaxK = 8192;       // unexpanded columns C*g

struct FusedLds {
    int a_off, b_off, tail_off, first_off, cursor_off, ent_off, total;
};
static FusedLds fused_lds(int BM, int BN, int ksteps_main, int tail_steps, int T) {
    FusedLds l;
    l.a_off = 0;
    l.b_off = 2 * BM * 64;
    l.tail_off = l.b_off + 2 * BN * 64;
    l.first_off = l.tail_off + tail_steps * BM * 64;
    l.cursor_off = l.first_off + (ksteps_main + 2) * 4;
    l.ent_off = l.cursor_off + (ksteps_main + 1) * 4;
    l.total = l.ent_off + (T > 0 ? T : 1) * 4;
    return l;
}

template <int BN, int BM, int NT, int WPE, int SETS>
__global__ __launch_bounds__(NT, WPE) void split_act_qgemm_kernel(
    const float* __restrict__ X, int64_t ldx, int M, int C, int g, int s,
    const int32_t* __restrict__ chan_src, const float* __restrict__ thr, float qmax,
    const int8_t* __restrict__ Wq, int64_t ldw, int N, int ksteps_main, int ksteps_all, int rem,
    const float* __restrict__ scale_w, float* __restrict__ scale_x_out, int32_t* __restrict__ acc_out,
    int64_t ldacc, float* __restrict__ Y, int64_t ldy, FusedLds L, int bm_stride) {
    // bm_stride: rows between consecutive workgroups' first rows (<= BM): a workgroup owns rows
    // row0 .. row0 + bm_stride - 1 and the rest of its BM rows are idle (nothing fetched or stored).
    // ksteps_main: whole 64-column steps of X; rem: the columns of X left over after them (< 64).
    // They and the appended columns form the steps ksteps_main .. ksteps_all-1, which are assembled
    // in LDS (`tail`): the left-over columns are quantized straight into its first step.
    constexpr int NW = NT / 64;
    constexpr int A_PER = BM * 16 / NT;        // 16-byte loads of X per thread and step (64 floats x BM rows)
    constexpr int WAVES_M = BM / 32, WAVES_N = NW / WAVES_M, WN = BN / WAVES_N, TN = WN / 32;
    static_assert(A_PER >= 1 && A_PER * NT == BM * 16 && WAVES_M * WAVES_N == NW && TN >= 1 && TN * 32 * WAVES_N == BN,
                  "the threads tile a step of X, the waves tile the outputs in 32 x 32 blocks");
    constexpr int B_SLOTS = BN * 4, B_PER = (B_SLOTS + NT - 1) / NT;
    static_assert(BN == 64 || BN == 128 || BN == 256, "64, 128 or 256 output columns");
    static_assert(NW * 8 * WN * 4 <= 2 * BM * 64 + 2 * BN * 64, "the epilogue's staging area is the operand buffers");

    extern __shared__ __align__(1024) int8_t flds[];
    int8_t* a_buf = flds + L.a_off;
    int8_t* b_buf = flds + L.b_off;
    int8_t* tail = flds + L.tail_off;
    int* first = reinterpret_cast<int*>(flds + L.first_off);     // [ksteps_main + 2]
    int* cursor = reinterpret_cast<int*>(flds + L.cursor_off);   // [ksteps_main + 1]
    int* ent = reinterpret_cast<int*>(flds + L.ent_off);         // [T]: (e << 6) | source column inside its step

    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int row0 = (int)blockIdx.x * bm_stride;
    const int row_end = row0 + bm_stride < M ? row0 + bm_stride : M;
    const int T = s * g, tail_steps = ksteps_all - ksteps_main;

    // A: the step's BM x 16 float4 numbered row-major; load i of thread t is number i*NT + t, so each
    // load instruction of a wave covers four rows' whole 256 bytes
    const float* a_src[A_PER];
    unsigned a_ok = 0;  // bit i: load i of this thread lies in a row the workgroup owns
    int a_dst[A_PER];   // byte offset of the resulting code dword inside an A buffer
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
        const int f = i * NT + tid, r = f >> 4, f4 = f & 15;
        int gr = row0 + r;
        if (gr < row_end) a_ok |= 1u << i;
        gr = gr < row_end ? gr : row_end - 1;          // rows past the workgroup's own are never fetched or stored
        a_src[i] = X + (int64_t)gr * ldx + f4 * 4;
        a_dst[i] = r * 64 + swz<64>(r, f4 >> 2) * 16 + (f4 & 3) * 4;
    }
    // B: 16-byte piece (slot & 3) of the step of weight row (slot >> 2)
    static_assert(B_PER * NT == B_SLOTS, "every thread moves the same number of weight pieces");
    const int8_t* b_src[B_PER];
    int b_dst[B_PER], b_piece[B_PER];
    const int b_pieces = (int)(ldw / 16);
#pragma unroll
    for (int u = 0; u < B_PER; ++u) {
        const int slot = u * NT + tid, n = slot >> 2, c = slot & 3;
        const int gn = col_clamp(n, N);
        b_src[u] = Wq + (int64_t)gn * ldw;
        b_piece[u] = c;
        b_dst[u] = n * 64 + swz<64>(n, c) * 16;
    }

    // SETS register sets in rotation: while one is processed, the next SETS-1 steps are on their way
    static_assert(SETS == 2 || SETS == 3, "one or two steps ahead");
    f32x4 av[SETS][A_PER];
    i32x4 bv[SETS][B_PER];
    auto load_step = [&](int kt, f32x4 (&a)[A_PER], i32x4 (&b)[B_PER]) {
        // Every lane issues the same loads at every step, whatever the step holds for it: a lane with
        // nothing to fetch (steps past the columns of X, pieces past a pitch, left-over columns that
        // do not exist) reads the 16 zero bytes instead, which costs one request per wave.  With no
        // branch around any load, the number of loads in flight is known at every wait, and the
        // waits let the two steps that are on their way stay on their way.
        const bool main_step = kt < ksteps_main, rest_step = kt == ksteps_main && rem > 0;
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int c0 = ((i * NT + tid) & 15) * 4;
            // left-over columns: a float4 that would cross the row's end starts four floats before
            // the end instead, and is shifted into place afterwards (nothing is read past the row)
            const bool ok = (a_ok >> i) & 1u;
            const bool whole = ok && (main_step || (rest_step && c0 + 3 < rem));
            const bool part = ok && rest_step && c0 < rem && !whole;
            const float* src = whole ? a_src[i] + (int64_t)kt * 64
                                     : (part ? a_src[i] + (int64_t)kt * 64 - c0 + (rem - 4)
                                             : reinterpret_cast<const float*>(zero_chunk));
            a[i] = *reinterpret_cast<const f32x4u*>(src);     // (shifted when it is used, not here)
        }
#pragma unroll
        for (int u = 0; u < B_PER; ++u) {
            const int piece = kt * 4 + b_piece[u];
            // a pitch may end inside the last K-step: what the row lacks counts as zero codes
            b[u] = *reinterpret_cast<const i32x4*>(kt < ksteps_all && piece < b_pieces ? b_src[u] + piece * 16
                                                                                       : zero_chunk);
        }
    };
    load_step(0, av[0], bv[0]);
    if (SETS == 3) load_step(1, av[1], bv[1]);

    // set-up behind the first requests: clear the appended steps, bucket the appended columns
    {
        i32x4 z = {0, 0, 0, 0};
        for (int o = tid; o < tail_steps * (BM * 64 / 16); o += NT) reinterpret_cast<i32x4*>(tail)[o] = z;
        for (int k = tid; k <= ksteps_main + 1; k += NT) first[k] = 0;
        __syncthreads();
        for (int e = tid; e < T; e += NT) {
            const int j = e / g, t = e - j * g;
            const int col = col_clamp(chan_src[C + j], C) * g + t;
            atomicAdd(&first[(col >> 6) + 1], 1);
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
            const int col = col_clamp(chan_src[C + j], C) * g + t;
            const int pos = atomicAdd(&cursor[col >> 6], 1);
            ent[pos] = (e << 6) | (col & 63);
        }
        // (the first step's barrier completes the table before anyone reads it)
    }

    const float Tx = *thr;
    const float inv = inv_step_of(Tx, qmax);
    if (scale_x_out != nullptr && blockIdx.x == 0 && tid == 0) {
        scale_x_out[0] = Tx;
        scale_x_out[1] = Tx / qmax;
    }

    i32x16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0;
    const int frag_row = lane & 31, frag_half = lane >> 5;

    auto process = [&](int kt, const f32x4 (&a)[A_PER], const i32x4 (&b)[B_PER]) {
        const int buf = kt & 1;
        int8_t* ab = a_buf + buf * (BM * 64);
        int8_t* bb = b_buf + buf * (BN * 64);
        const bool main_step = kt < ksteps_main;
        const bool rest_step = kt == ksteps_main && rem > 0;     // holds the left-over columns of X
        if (main_step || rest_step) {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const unsigned q4 = pack4(code_bits(a[i][0], inv, qmax), code_bits(a[i][1], inv, qmax),
                                          code_bits(a[i][2], inv, qmax), code_bits(a[i][3], inv, qmax));
                if (main_step) {
                    *reinterpret_cast<unsigned*>(ab + a_dst[i]) = q4;
                } else {
                    // into the first assembled step, byte by byte where the dword also holds copies.
                    // A float4 that straddled the row's end was fetched as columns rem-4 .. rem-1:
                    // this lane's column c0 + e is its element c0 + e - (rem - 4)
                    const int c0 = ((i * NT + tid) & 15) * 4;
                    if (c0 + 3 < rem) {
                        *reinterpret_cast<unsigned*>(tail + a_dst[i]) = q4;
                    } else {
                        const int d = c0 - (rem - 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (c0 + e < rem) tail[a_dst[i] + e] = (int8_t)((q4 >> (8 * (e + d))) & 0xFFu);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < B_PER; ++u) *reinterpret_cast<i32x4*>(bb + b_dst[u]) = b[u];
        __syncthreads();
        const int8_t* am = main_step ? ab : tail + (kt - ksteps_main) * (BM * 64);
        if (main_step || rest_step) {
            // the copies whose sources this step holds: one byte per (copy, row), to expanded column
            // C*g + e, which is column rem + e of the assembled steps
            const int e0 = first[kt], n = first[kt + 1] - e0;
            for (int idx = tid; idx < n * BM; idx += NT) {
                const int q = idx / BM, r = idx - q * BM;
                const int en = ent[e0 + q], e = rem + (en >> 6), c = en & 63;
                const int8_t code = am[r * 64 + swz<64>(r, c >> 4) * 16 + (c & 15)];
                const int te = e & 63;
                tail[(e >> 6) * (BM * 64) + r * 64 + swz<64>(r, te >> 4) * 16 + (te & 15)] = code;
            }
            if (rest_step) __syncthreads();    // this very step may hold some of those copies
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int ra = wm * 32 + frag_row;
            const i32x4 fa = *reinterpret_cast<const i32x4*>(&am[ra * 64 + swz<64>(ra, ks * 2 + frag_half) * 16]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int rb = wn * WN + j * 32 + frag_row;
                const i32x4 fb = *reinterpret_cast<const i32x4*>(&bb[rb * 64 + swz<64>(rb, ks * 2 + frag_half) * 16]);
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc[j], 0, 0, 0);
            }
        }
    };

    for (int kt0 = 0; kt0 < ksteps_all; kt0 += SETS) {
#pragma unroll
        for (int p = 0; p < SETS; ++p) {
            const int kt = kt0 + p;
            if (kt < ksteps_all) {
                load_step(kt + SETS - 1, av[(p + SETS - 1) % SETS], bv[(p + SETS - 1) % SETS]);
                process(kt, av[p], bv[p]);
            }
        }
    }
    __syncthreads();   // the operand buffers are dead: they become the staging area

    int32_t* stage = reinterpret_cast<int32_t*>(flds + wave * (8 * WN * 4));
    const float scale = (Tx / qmax) * scale_w[1];
    const bool vec_y = (reinterpret_cast<uintptr_t>(Y) % 16 == 0) && (ldy % 4 == 0);
    const bool vec_a = acc_out != nullptr && (reinterpret_cast<uintptr_t>(acc_out) % 16 == 0) && (ldacc % 4 == 0);
    const Requant none{};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                stage[((lane >> 5) * 4 + e) * WN + j * 32 + (lane & 31)] = acc[j][q * 4 + e];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        emit_staged_rows<8, WN>(stage, lane, row0 + wm * 32 + q * 8, wn * WN, wn * WN, row_end, N, scale, Y, ldy,
                                acc_out, ldacc, vec_y, vec_a, none, 0.0f, nullptr, 0, false);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// Where the one launch is ahead of the two (measured on the same shapes): from 256 columns of X
// on.  With 64 the pass over X is short either way and the output dominates.
bool split_act_qgemm_pays(int64_t M, int C, int g, int s, int64_t N, int64_t ldx) {
    return split_act_qgemm_fits(M, C, g, s, N, ldx) && (int64_t)C * g >= 128;
}

bool split_act_qgemm_fits(int64_t M, int C, int g, int s, int64_t N, int64_t ldx) {
    const int64_t K = (int64_t)C * g, T = (int64_t)s * g;
    (void)ldx;
    return M >= 1 && M <= 0x7FFFFFFF - kFusedMaxBM && K >= 64 && K <= kFusedMaxK && T <= kFusedMaxTail && N >= 1 &&
           N <= 256;
}

template <int BN, int BM, int NT, int WPE, int SETS>
static hipError_t run_split_act_qgemm(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                      const int32_t* chan_src, const float* thr, float qmax, const int8_t* Wq,
                                      int64_t ldw, int64_t N, int64_t Kexp, const float* scale_w,
                                      float* scale_x_out, int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                                      hipStream_t stream) {
    const int ksteps_main = (int)((int64_t)C * g / 64), ksteps_all = (int)ceil_div(Kexp, 64);
    const int rem = (int)((int64_t)C * g - (int64_t)ksteps_main * 64);
    const FusedLds L = fused_lds(BM, BN, ksteps_main, ksteps_all - ksteps_main, s * g);
    if (L.total > kWholeKMaxLds) return hipErrorInvalidValue;
    static std::atomic<bool> opted_in[kMaxDevices];
    if (L.total > 65536) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        if (!opted_in[dev].load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&split_act_qgemm_kernel<BN, BM, NT, WPE, SETS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWholeKMaxLds);
            if (e != hipSuccess) return e;
            opted_in[dev].store(true, std::memory_order_release);
        }
    }
    // When the row tiles would not even fill the chip's workgroup slots once, fewer rows per
    // workgroup and a workgroup in every slot: the pass is bound by what a compute unit can draw
    // from memory, so idle matrix rows cost nothing and idle compute units do (392 tiles of 128
    // rows on 512 slots: 134 -> 122 us on the 256-channel 3x3 layers at 14 x 14, batch 256).
    int64_t stride = BM;
    {
        int wpc = (int)(kWholeKMaxLds / L.total);
        wpc = wpc > WPE ? WPE : (wpc < 1 ? 1 : wpc);
        const int64_t slots = (int64_t)compute_units() * wpc;
        const int ts = tuning().fused_stride;
        if (ts > 0 && ts <= BM) stride = ts;
        else if (ts != 0 && ceil_div(M, BM) < slots) stride = ceil_div(M, slots);
        if (stride < BM / 2) stride = BM / 2;      // (never more than half of a tile idle)
    }
    return launch_kernel(kTimeGemm, split_act_qgemm_kernel<BN, BM, NT, WPE, SETS>, dim3((unsigned)ceil_div(M, stride)),
                         dim3(NT), (unsigned)L.total, stream, X, ldx, (int)M, C, g, s, chan_src, thr, qmax,
                         Wq, ldw, (int)N, ksteps_main, ksteps_all, rem, scale_w, scale_x_out, acc_out, ldacc, Y, ldy, L,
                         (int)stride);
}

hipError_t launch_split_act_qgemm(const float* X, int64_t ldx, int64_t M, int C, int g, int s,
                                  const int32_t* chan_src, const float* thr, float qmax, const int8_t* Wq,
                                  int64_t ldw, int64_t N, int64_t Kexp, const float* scale_w, float* scale_x_out,
                                  int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream) {
    if (!split_act_qgemm_fits(M, C, g, s, N, ldx)) return hipErrorInvalidValue;
#define OCS_FUSED_ARGS X, ldx, M, C, g, s, chan_src, thr, qmax, Wq, ldw, N, Kexp, scale_w, scale_x_out, acc_out, ldacc, Y, ldy, stream
    // Measured on the paper's layer shapes at batch 256.  Up to 128 output columns: workgroups of 64
    // rows on 4 waves, three or four of them per compute unit, each with its own barriers (10-20 %
    // ahead of 128-row ones).  256 columns: the weight codes a workgroup pulls per step weigh as much
    // as 64 rows of X, and 128 rows on 8 waves are ahead, except on very tall X, where two 64-row
    // workgroups per compute unit win.  One step of look-ahead everywhere: a second one was level or
    // behind (its registers cost a workgroup per compute unit).
    const int v = tuning().fused_variant;     // tests: 1 / 2 force the 64- / 128-row shape for N > 128
    if (N <= 64) return run_split_act_qgemm<64, 64, 256, 4, 2>(OCS_FUSED_ARGS);
    if (N <= 128) return run_split_act_qgemm<128, 64, 256, 3, 2>(OCS_FUSED_ARGS);
    if (v == 1 || (v != 2 && M >= 131072)) return run_split_act_qgemm<256, 64, 512, 4, 2>(OCS_FUSED_ARGS);
    return run_split_act_qgemm<256, 128, 512, 2, 2>(OCS_FUSED_ARGS);
#undef OCS_FUSED_ARGS
}


// Dynamic LDS of a whole-K launch: operands (or the epilogue's staging area, if larger) and,
// when the output goes to the next layer as codes with copies, the table of those copies
// behind them (*dup_off = its byte offset, 0 = none).
template <int BM, int BN, int WAVES_M, int WAVES_N>
static int64_t wholek_lds_bytes(int64_t Kpad, const Requant& rq, int* dup_off = nullptr) {
    const int64_t operands = (Kpad / 64) * (BM + BN) * 64;
    const int64_t staging = (int64_t)WAVES_M * WAVES_N * 8 * (BN / WAVES_N) * 4;
    int64_t lds = operands > staging ? operands : staging;
    int off = 0;
    if (rq.Yq != nullptr && rq.s_next > 0) {
        off = (int)round_up(lds, 16);
        lds = off + (kDupCap + 1) * 4;
    }
    if (dup_off) *dup_off = off;
    return lds;
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
static hipError_t run_wholek(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw,
                             int64_t M, int64_t N, int64_t Kpad, const float* scale_x,
                             const float* scale_w, int32_t* acc_out, int64_t ldacc, float* Y,
                             int64_t ldy, hipStream_t stream, const Requant& rq) {
    int dup_off = 0;
    const int64_t lds = wholek_lds_bytes<BM, BN, WAVES_M, WAVES_N>(Kpad, rq, &dup_off);
    if (Kpad < 64 || Kpad % 64 != 0 || lds > kWholeKMaxLds) return hipErrorInvalidValue;
    // more than 64 KB of dynamic LDS has to be opted into, once per kernel and device (setting
    // it twice from two threads is harmless)
    static std::atomic<bool> opted_in[kMaxDevices];
    int dev = 0;
    if (lds > 65536) {
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        if (!opted_in[dev].load(std::memory_order_acquire)) {
            e = hipFuncSetAttribute(
                reinterpret_cast<const void*>(&qgemm_wholek_kernel<BM, BN, WAVES_M, WAVES_N>),
                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kWholeKMaxLds);
            if (e != hipSuccess) return e;
            opted_in[dev].store(true, std::memory_order_release);
        }
    }
    const int64_t tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
    const int64_t total = tiles_m * tiles_n;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;   // one workgroup per tile: grid.x
    return launch_kernel(kTimeGemm, qgemm_wholek_kernel<BM, BN, WAVES_M, WAVES_N>,
                         dim3((unsigned)total), dim3(WAVES_M * WAVES_N * 64), (unsigned)lds, stream,
                         Xq, ldx, Wq, ldw, (int)M, (int)N, (int)(Kpad / 64), scale_x, scale_w,
                         acc_out, ldacc, Y, ldy, (int)tiles_n, (unsigned)total, dup_off, rq);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NBUF, bool MASK = false>
static hipError_t run_dma(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                          int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                          int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                          hipStream_t stream, const Requant& rq) {
    // without MASK the kernel walks whole K-steps of every row
    if (!MASK && (ldx < Kpad || ldw < Kpad)) return hipErrorInvalidValue;
    // the kernel clamps its K index to ksteps - 1: it must never be launched with no K-step
    if (Kpad < BK || Kpad % BK != 0) return hipErrorInvalidValue;
    const int64_t tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
    const int64_t total = tiles_m * tiles_n;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;   // one workgroup per tile: grid.x
    return launch_kernel(kTimeGemm, qgemm_dma_kernel<BM, BN, WAVES_M, WAVES_N, BK, NBUF, false, false, MASK>,
                         dim3((unsigned)total), dim3(WAVES_M * WAVES_N * 64), 0, stream, Xq, ldx, Wq, ldw, (int)M,
                         (int)N, (int)(Kpad / BK), scale_x, scale_w, acc_out, ldacc, Y, ldy,
                         (int)tiles_n, (unsigned)total, ConvGeom{}, rq, SplitK{});
}

// Arrival counters of the K split: part of the library's device image (zero when the module is
// loaded, and every launch leaves the counters it used at zero again), one copy per GPU.  A launch
// takes one slot of kSplitSlotTiles counters, slots handed out in turn, so that launches on
// different streams do not share counters unless more than kSplitSlots of them are in flight on
// one GPU.  In host code the array's name is only a handle: the device address is looked up once
// per device and only that address goes to a launch.
constexpr int kSplitSlotTiles = 128;
constexpr int kSplitSlots = 512;
static __device__ unsigned splitk_counters[kSplitSlotTiles * kSplitSlots];

static hipError_t splitk_counter_slot(unsigned** out) {
    static std::atomic<unsigned*> addr[kMaxDevices];
    static std::atomic<unsigned> cursor[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    unsigned* p = addr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(splitk_counters));
        if (e != hipSuccess) return e;
        if (sym == nullptr) return hipErrorInvalidSymbol;
        p = static_cast<unsigned*>(sym);
        addr[dev].store(p, std::memory_order_release);
    }
    const unsigned slot = cursor[dev].fetch_add(1u, std::memory_order_relaxed) % (unsigned)kSplitSlots;
    *out = p + (size_t)slot * kSplitSlotTiles;
    return hipSuccess;
}

// The split kernel's tile is 256 x 256 (64-byte K-steps, ring of four).
constexpr int kSplitBM = 256, kSplitBN = 256;

// 0 when the shape cannot be split this way (more tiles than a counter slot holds, or fewer than
// one K-step per part).
size_t qgemm_split_workspace_bytes(int64_t M, int64_t N, int64_t Kpad, int parts) {
    const int64_t tiles = ceil_div(M, kSplitBM) * ceil_div(N, kSplitBN);
    if (parts < 2 || parts > 16 || tiles > kSplitSlotTiles || Kpad / 64 < parts) return 0;
    return (size_t)tiles * parts * kSplitBM * kSplitBN * sizeof(int32_t);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NBUF>
static hipError_t run_dma_split(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                                int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                                int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream,
                                const Requant& rq, int parts, void* partials) {
    if (Kpad < BK || Kpad % BK != 0 || parts < 2 || Kpad / BK < parts) return hipErrorInvalidValue;
    const int64_t tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
    const int64_t total = tiles_m * tiles_n;
    if (total > kSplitSlotTiles) return hipErrorInvalidValue;
    SplitK sk;
    sk.partials = static_cast<int32_t*>(partials);
    sk.parts = parts;
    hipError_t e = splitk_counter_slot(&sk.counters);
    if (e != hipSuccess) return e;
    return launch_kernel(kTimeGemm, qgemm_dma_kernel<BM, BN, WAVES_M, WAVES_N, BK, NBUF, false, true>,
                         dim3((unsigned)(total * parts)), dim3(WAVES_M * WAVES_N * 64), 0, stream, Xq, ldx, Wq,
                         ldw, (int)M, (int)N, (int)(Kpad / BK), scale_x, scale_w, acc_out, ldacc, Y, ldy,
                         (int)tiles_n, (unsigned)total, ConvGeom{}, rq, sk);
}

// The same kernel with the lowering of a convolution done by its A-operand loader.
template <int BM, int BN, int WAVES_M, int WAVES_N, int NBUF>
static hipError_t run_dma_conv(const int8_t* Aq, const int8_t* Wt, int64_t ldw, int64_t M, int64_t N,
                               int64_t Kpad, const ConvGeom& cg, const float* scale_x,
                               const float* scale_w, int32_t* acc_out, int64_t ldacc, float* Y,
                               int64_t ldy, hipStream_t stream, const Requant& rq) {
    constexpr int BK = 64;
    if (Kpad < BK || Kpad % BK != 0 || cg.ldc % 16 != 0 || cg.cpp < 1) return hipErrorInvalidValue;
    const int64_t tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
    const int64_t total = tiles_m * tiles_n;
    if (total > 0x7FFFFFFF) return hipErrorInvalidValue;   // one workgroup per tile: grid.x
    return launch_kernel(kTimeGemm, qgemm_dma_kernel<BM, BN, WAVES_M, WAVES_N, BK, NBUF, true>,
                         dim3((unsigned)total), dim3(WAVES_M * WAVES_N * 64), 0, stream, Aq, cg.ldc, Wt,
                         ldw, (int)M, (int)N, (int)(Kpad / BK), scale_x, scale_w, acc_out, ldacc, Y,
                         ldy, (int)tiles_n, (unsigned)total, cg, rq, SplitK{});
}

hipError_t launch_qconv(const int8_t* Aq, int64_t ldc, int B, int H, int W, int kh, int kw, int stride,
                        int pad, const int8_t* Wt, int64_t ldw, int64_t N, const float* scale_x,
                        const float* scale_w, int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                        hipStream_t stream, const Requant& rq) {
    ConvGeom cg;
    cg.Ho = (H + 2 * pad - kh) / stride + 1;
    cg.Wo = (W + 2 * pad - kw) / stride + 1;
    cg.H = H;
    cg.W = W;
    cg.kh = kh;
    cg.kw = kw;
    cg.cpp = (int)(ldc / 16);
    cg.stride = stride;
    cg.pad = pad;
    cg.ldc = ldc;
    cg.zero = Wt + N * ldw;            // the row of zeros that follows the N weight rows
    const int64_t M = (int64_t)B * cg.Ho * cg.Wo;
    const int64_t Kpad = ldw;          // kh*kw*ldc rounded up to a whole K-step
    if (Kpad < (int64_t)kh * kw * ldc) return hipErrorInvalidValue;
    int tile = tuning().gemm_tile;
    // measured on the stem and the 3x3 layers of the paper's networks: the 128x128 tile is level
    // with or ahead of the larger ones (the loader's per-lane tap bookkeeping grows with the rows
    // a lane loads; a 128-byte K-step, which doubles them, was 15-90 % slower) and, from 64
    // output channels on, ahead of the 128x64 one as well
    if (tile < 0) tile = N < 64 ? 6 : 9;
#define OCS_CONV_ARGS Aq, Wt, ldw, M, N, Kpad, cg, scale_x, scale_w, acc_out, ldacc, Y, ldy, stream, rq
    switch (tile) {
        case 6: return run_dma_conv<128, 64, 2, 2, 6>(OCS_CONV_ARGS);
        case 7: return run_dma_conv<64, 64, 2, 2, 6>(OCS_CONV_ARGS);
        case 10: return run_dma_conv<256, 128, 4, 2, 4>(OCS_CONV_ARGS);
        case 12: return run_dma_conv<256, 256, 2, 4, 4>(OCS_CONV_ARGS);
        default: return run_dma_conv<128, 128, 4, 2, 4>(OCS_CONV_ARGS);
    }
#undef OCS_CONV_ARGS
}

// Channel-major codes [N, ldq] (column j*g + t) -> tap-major [N + 1, ldt] (column t*ldc + j,
// zero for j >= E and for columns past g*ldc), the extra row all zeros.  One lane per byte quad.
__global__ __launch_bounds__(kThreads) void tap_major_kernel(const int8_t* __restrict__ Wq, int64_t ldq,
                                                             int64_t N, int E, int g, int64_t ldc,
                                                             int64_t ldt, int8_t* __restrict__ Wt) {
    const int64_t quads_per_row = ldt / 4;
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o >= (N + 1) * quads_per_row) return;
    const int64_t n = o / quads_per_row;
    const int64_t k = (o - n * quads_per_row) * 4;     // ldc % 4 == 0: a quad stays inside one tap
    const int t = (int)(k / ldc);
    const int j0 = (int)(k - (int64_t)t * ldc);
    unsigned packed = 0;
    if (n < N && t < g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = j0 + e;
            const int code = j < E ? Wq[n * ldq + (int64_t)j * g + t] : 0;
            packed |= ((unsigned)code & 0xFFu) << (8 * e);
        }
    }
    reinterpret_cast<unsigned*>(Wt)[o] = packed;
}

hipError_t launch_tap_major(const int8_t* Wq, int64_t ldq, int64_t N, int E, int g, int64_t ldc,
                            int8_t* Wt, hipStream_t stream) {
    const int64_t ldt = round_up((int64_t)g * ldc, 64);
    const int64_t total = (N + 1) * (ldt / 4);
    if (ceil_div(total, kThreads) > 0x7FFFFFFF) return hipErrorInvalidValue;   // one lane per byte quad: grid.x
    tap_major_kernel<<<dim3((unsigned)ceil_div(total, kThreads)), kThreads, 0, stream>>>(Wq, ldq, N, E, g,
                                                                                       ldc, ldt, Wt);
    return hipGetLastError();
}

#define OCS_GEMM_ARGS Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w, acc_out, ldacc, Y, ldy, stream, rq
#define OCS_GEMM_ARGS128 Xq, ldx, Wq, ldw, M, N, K128, scale_x, scale_w, acc_out, ldacc, Y, ldy, stream, rq

hipError_t launch_qgemm(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                        int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                        int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                        hipStream_t stream, const Requant& rq) {
    int tile = tuning().gemm_tile;
    // A pitch that is not a whole number of 64-byte K-steps, or shorter than the K extent rounded
    // up to one (allowed up to 320 bytes of K), is something only the whole-K kernel walks.
    const bool ring_ok = ldx % 64 == 0 && ldw % 64 == 0 && ldx >= Kpad && ldw >= Kpad;
    if (!ring_ok) {
        if (Kpad > 320) return hipErrorInvalidValue;
        // (the 128 x 128 ring variant checks its requests against the pitch for this case: a very
        // wide N is better served by the ring kernel's tile order, see below)
        if (tile == 9 || (tile < 0 && N >= 1024))
            return run_dma<128, 128, 4, 2, 64, 4, true>(OCS_GEMM_ARGS);
        if (tile != 16 && tile != 17 && tile != 18 && tile != 19) tile = N <= 64 ? 17 : (N >= 512 ? (Kpad <= 192 ? 17 : 19) : 16);
    }
    if (tile < 0) {
        // Measured on MI355X over the layer shapes of the paper's networks.  What a CU can draw is
        // set by the line requests its L1 can have outstanding times their latency, so requests
        // count, not bytes: the largest tile that still gives most CUs a workgroup wins, a K-step
        // of one whole 128-byte line per row beats two half-line steps, and workgroups of 8 waves
        // beat 4.  Up to 320 bytes of K the layer is a stream of output rows and the whole-K kernel
        // wins (1.2-1.5x), except that a very wide N is better served by the ring kernel's tile
        // order (one L2 fill of an X row panel for all its N tiles).  With N >= 256 and enough
        // tiles, 256 columns per tile halve the reads of X.
        const int64_t t256 = ceil_div(M, 256) * ceil_div(N, 128);
        const int64_t t128 = ceil_div(M, 128) * ceil_div(N, 128);
        const int64_t t256sq = ceil_div(M, 256) * ceil_div(N, 256);
        if (Kpad <= 320) tile = N <= 64 ? 17 : (N >= 1024 ? 9 : (N >= 512 ? (Kpad <= 192 ? 17 : 19) : 16));   // (512 outputs from
                                        // 128 channels: the 128 x 64 tile, 70 against 83 us at M = 200,704)
        else if (N <= 64) tile = 24;    // 128 x 64 with whole-line (128-byte) K-steps: 134 against 155 us on
                                        // the 64 -> 64 3x3 layers at M = 802,816
        else if (N >= 256 && t256sq >= 192 && Kpad >= 1024) tile = 12;
        else if (N >= 1024 && Kpad < 1024) tile = 9;     // (launched alone on cold operands the 256 x 256 tile
                                                         // is ahead here; behind the pass that wrote the codes
                                                         // it is 7-18 % behind)
        else if (N >= 512 && t256sq >= 512) tile = 12;
        else if (N >= 512 && t256 >= 128 && t256 < 256 && Kpad >= 4096) tile = 25;   // fewer tiles than compute units and a very long K:
                                        // 128 x 256 (X rows asked for by two tiles, not four; 43-46 against 45-47 us
                                        // on the 512 -> 512 3x3 layers at M = 12544; behind at half that K)
        else if (t256 >= 128) tile = 11;                 // N = 256 with K below 1024 included (89 against 92 us)
        else if (t128 >= 48) tile = 23;   // 128-byte K-steps when the operands allow them
        else tile = 6;
    }
    // A 128-byte K-step needs a K extent that is a multiple of 128.  The extent is the codes
    // rounded up to 64; when both leading dimensions hold 64 bytes more, those are zero padding
    // on both operands (the producers' contract) and the walk may include them.
    const int64_t K128 = round_up(Kpad, 128);
    const bool k128 = K128 == Kpad || (ldx >= K128 && ldw >= K128);
    // Tile variants by id (the dispatcher above picks 6, 9, 11, 12, 16, 17, 19, 23, 24 or 25; the others
    // are kept selectable because the parity tests run every kernel family through them).
    switch (tile) {
        case 6: return run_dma<128, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS);
        case 7: return run_dma<64, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS);
        case 9: return run_dma<128, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS);    // 8 waves
        case 10: return run_dma<256, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS);   // 8 waves
        case 11: return k128 ? run_dma<256, 128, 4, 2, 128, 3>(OCS_GEMM_ARGS128)  // 8 waves
                             : run_dma<256, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS);
        case 12: return run_dma<256, 256, 2, 4, 64, 4>(OCS_GEMM_ARGS);   // 8 waves
        case 14: return run_dma<256, 256, 4, 4, 64, 4>(OCS_GEMM_ARGS);   // 16 waves
        // whole-K variants; a K extent too long for them falls back to a ring variant
#define OCS_WHOLEK(BM_, BN_, WM_, WN_, FALLBACK)                                                   \
    (wholek_lds_bytes<BM_, BN_, WM_, WN_>(Kpad, rq) <= kWholeKMaxLds                                   \
         ? run_wholek<BM_, BN_, WM_, WN_>(OCS_GEMM_ARGS)                                            \
         : FALLBACK)
        case 16: return OCS_WHOLEK(128, 128, 4, 2, (run_dma<128, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS)));
        case 17: return OCS_WHOLEK(128, 64, 4, 1, (run_dma<128, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS)));
        case 18: return OCS_WHOLEK(64, 64, 2, 2, (run_dma<64, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS)));
        case 19: return OCS_WHOLEK(128, 256, 2, 4, (run_dma<128, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS)));
#undef OCS_WHOLEK
        case 23: return k128 ? run_dma<128, 128, 4, 2, 128, 3>(OCS_GEMM_ARGS128)
                             : run_dma<128, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS);
        case 24: return k128 ? run_dma<128, 64, 2, 2, 128, 3>(OCS_GEMM_ARGS128)
                             : run_dma<128, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS);
        case 25: return k128 ? run_dma<128, 256, 2, 4, 128, 3>(OCS_GEMM_ARGS128)
                             : run_dma<256, 128, 4, 2, 64, 4>(OCS_GEMM_ARGS);
        default: return run_dma<64, 64, 2, 2, 64, 6>(OCS_GEMM_ARGS);
    }
}

hipError_t launch_qgemm_split(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                              int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                              int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream,
                              int parts, void* partials) {
    return run_dma_split<kSplitBM, kSplitBN, 2, 4, 64, 4>(Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w,
                                                         acc_out, ldacc, Y, ldy, stream, Requant{}, parts,
                                                         partials);
}

}  // namespace ocs
