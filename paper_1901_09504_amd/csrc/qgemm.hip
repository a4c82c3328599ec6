// The expanded layer (Eq. 2 over the expanded channel set) on int8 codes: an NT GEMM
// acc[i,n] = sum_k Xq[i,k] * Wq[n,k] on the matrix cores (v_mfma_i32_32x32x32_i8, int32
// accumulation, exact), with the trailing scale factors of Eq. 1 applied in the epilogue.
//
// Both operands are K-contiguous, so a lane's MFMA operand is 16 consecutive bytes of one
// row.  A workgroup of 4 waves computes a BM x BN tile; per K-step of 64 bytes the BM + BN
// row segments are staged in LDS (two buffers; the global loads of step k+1 are in flight in
// registers while step k is multiplied).  LDS rows are 64 bytes = four 16-byte chunks; the
// chunk index is XOR-swizzled with the row so that the 16-byte reads of consecutive rows
// fall in different banks.  K is padded with zero codes to a multiple of 64 by the producers,
// so the K loop has no tail; zeros add nothing to an integer sum.
#include "ocs_internal.h"

namespace ocs {

__device__ __forceinline__ int swz(int row, int chunk) {
    return chunk ^ (((row >> 2) & 3) ^ (row & 2));
}

// Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber them so
// that consecutive tile ids (which share an X row panel) run on the same XCD.
__device__ __forceinline__ unsigned xcd_remap(unsigned w, unsigned total) {
    const unsigned q = total / 8, r = total % 8;
    const unsigned xcd = w % 8, local = w / 8;
    return xcd * q + (xcd < r ? xcd : r) + local;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int P>
__global__ __launch_bounds__(kThreads) void qgemm_kernel(
    const int8_t* __restrict__ Xq, int64_t ldx, const int8_t* __restrict__ Wq, int64_t ldw, int M,
    int N, int ktiles, const float* __restrict__ scale_x, const float* __restrict__ scale_w,
    int32_t* __restrict__ acc_out, int64_t ldacc, float* __restrict__ Y, int64_t ldy, int tiles_n,
    unsigned total_tiles) {
    static_assert(WAVES_M * WAVES_N == kThreads / 64, "4 waves");
    static_assert(P % 2 == 0, "the LDS buffer index must be static in the unrolled loop");
    constexpr int BK = 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // 32x32 MFMA tiles per wave
    constexpr int A_CHUNKS = BM * 4 / kThreads, B_CHUNKS = BN * 4 / kThreads;
    static_assert(A_CHUNKS >= 1 && B_CHUNKS >= 1, "tile too small");

    __shared__ __align__(16) int8_t lds_a[2][BM * BK];
    __shared__ __align__(16) int8_t lds_b[2][BN * BK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    const unsigned tile = xcd_remap(blockIdx.x, total_tiles);
    const int bm = (int)(tile / tiles_n), bn = (int)(tile % tiles_n);
    const int row0 = bm * BM, col0 = bn * BN;

    // staging: chunk q = tid + u*256 -> tile row q/4, 16-byte chunk q%4
    const int8_t* a_src[A_CHUNKS];
    const int8_t* b_src[B_CHUNKS];
    int a_dst[A_CHUNKS], b_dst[B_CHUNKS];
#pragma unroll
    for (int u = 0; u < A_CHUNKS; ++u) {
        int q = tid + u * kThreads, r = q >> 2, c = q & 3;
        int gr = row0 + r;
        gr = gr < M ? gr : M - 1;  // rows past the edge re-read the last row; never stored
        a_src[u] = Xq + (int64_t)gr * ldx + c * 16;
        a_dst[u] = r * BK + swz(r, c) * 16;
    }
#pragma unroll
    for (int u = 0; u < B_CHUNKS; ++u) {
        int q = tid + u * kThreads, r = q >> 2, c = q & 3;
        int gr = col0 + r;
        gr = gr < N ? gr : N - 1;
        b_src[u] = Wq + (int64_t)gr * ldw + c * 16;
        b_dst[u] = r * BK + swz(r, c) * 16;
    }

    // P K-steps of both operands are in flight in registers at any time: a workgroup alone
    // on its CU must cover the whole memory latency with its own outstanding loads.  Loads are
    // unconditional (the K index is clamped to the last step, whose data is then simply
    // fetched again) so that the unrolled loop body is straight-line code and the wait before
    // each LDS write covers only the oldest stage, not every load in flight.
    i32x4 a_reg[P][A_CHUNKS], b_reg[P][B_CHUNKS];
    auto fetch = [&](int slot_kt, i32x4 (&ar)[A_CHUNKS], i32x4 (&br)[B_CHUNKS]) {
        const int kl = slot_kt < ktiles ? slot_kt : ktiles - 1;
        const int64_t koff = (int64_t)kl * BK;
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u)
            ar[u] = *reinterpret_cast<const i32x4*>(a_src[u] + koff);
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u)
            br[u] = *reinterpret_cast<const i32x4*>(b_src[u] + koff);
    };
#pragma unroll
    for (int p = 0; p < P; ++p) fetch(p, a_reg[p], b_reg[p]);

    i32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // operand fetch: lane -> row lane%32 of a 32-row MFMA tile, K bytes (lane/32)*16 .. +15 of
    // a 32-byte K slice.  A and B use the same mapping, so the pairing of K bytes is
    // consistent whatever order the hardware assigns to them inside the slice.
    const int frag_row = lane & 31, frag_half = lane >> 5;

    // One K-step: registers -> LDS buffer `buf`, barrier, refill the registers, multiply.
    // One barrier per step suffices: a wave that arrives at it has finished reading the other
    // buffer (previous step), so that buffer may be overwritten right after the next barrier.
    auto step = [&](int buf, i32x4 (&ar)[A_CHUNKS], i32x4 (&br)[B_CHUNKS], int refill_kt,
                    bool refill) {
#pragma unroll
        for (int u = 0; u < A_CHUNKS; ++u)
            *reinterpret_cast<i32x4*>(&lds_a[buf][a_dst[u]]) = ar[u];
#pragma unroll
        for (int u = 0; u < B_CHUNKS; ++u)
            *reinterpret_cast<i32x4*>(&lds_b[buf][b_dst[u]]) = br[u];
        __syncthreads();
        if (refill) fetch(refill_kt, ar, br);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            i32x4 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int r = wm * WM + i * 32 + frag_row;
                af[i] = *reinterpret_cast<const i32x4*>(
                    &lds_a[buf][r * BK + swz(r, ks * 2 + frag_half) * 16]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int r = wn * WN + j * 32 + frag_row;
                bf[j] = *reinterpret_cast<const i32x4*>(
                    &lds_b[buf][r * BK + swz(r, ks * 2 + frag_half) * 16]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0,
                                                                     0, 0);
        }
    };

    int kt0 = 0;
    for (; kt0 + P <= ktiles; kt0 += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) step(p & 1, a_reg[p], b_reg[p], kt0 + p + P, true);
    }
    // the last ktiles % P steps; their data is already in the registers
#pragma unroll
    for (int p = 0; p < P; ++p)
        if (kt0 + p < ktiles) step(p & 1, a_reg[p], b_reg[p], 0, false);

    // epilogue: accumulator register v of lane l holds row (v/4)*8 + (l/32)*4 + v%4 and
    // column l%32 of its 32x32 tile
    const float scale = scale_x[1] * scale_w[1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int c = col0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = row0 + wm * WM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (r < M && c < N) {
                    const int a = acc[i][j][v];
                    Y[(int64_t)r * ldy + c] = (float)a * scale;
                    if (acc_out) acc_out[(int64_t)r * ldacc + c] = a;
                }
            }
        }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int P>
static hipError_t run(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                      int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                      int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy, hipStream_t stream) {
    const int64_t tiles_m = ceil_div(M, BM), tiles_n = ceil_div(N, BN);
    const int64_t total = tiles_m * tiles_n;
    qgemm_kernel<BM, BN, WAVES_M, WAVES_N, P><<<(unsigned)total, kThreads, 0, stream>>>(
        Xq, ldx, Wq, ldw, (int)M, (int)N, (int)(Kpad / 64), scale_x, scale_w, acc_out, ldacc, Y,
        ldy, (int)tiles_n, (unsigned)total);
    return hipGetLastError();
}

#define OCS_GEMM_ARGS Xq, ldx, Wq, ldw, M, N, Kpad, scale_x, scale_w, acc_out, ldacc, Y, ldy, stream

hipError_t launch_qgemm(const int8_t* Xq, int64_t ldx, const int8_t* Wq, int64_t ldw, int64_t M,
                        int64_t N, int64_t Kpad, const float* scale_x, const float* scale_w,
                        int32_t* acc_out, int64_t ldacc, float* Y, int64_t ldy,
                        hipStream_t stream) {
    int tile = tuning().gemm_tile;
    if (tile < 0) {
        // enough tiles to cover 256 CUs at least twice, else smaller tiles
        const int64_t t128 = ceil_div(M, 128) * ceil_div(N, 128);
        tile = t128 >= 512 ? 0 : 1;
        if (N <= 64) tile = 2;
    }
    switch (tile) {
        case 0: return run<128, 128, 2, 2, 6>(OCS_GEMM_ARGS);
        case 1: return run<128, 64, 2, 2, 8>(OCS_GEMM_ARGS);
        case 2: return run<128, 64, 4, 1, 8>(OCS_GEMM_ARGS);
        case 3: return run<64, 128, 2, 2, 8>(OCS_GEMM_ARGS);
        case 4: return run<64, 256, 1, 4, 6>(OCS_GEMM_ARGS);
        case 5: return run<128, 128, 2, 2, 2>(OCS_GEMM_ARGS);
        case 6: return run<128, 64, 2, 2, 4>(OCS_GEMM_ARGS);
        default: return run<64, 64, 2, 2, 8>(OCS_GEMM_ARGS);
    }
}

}  // namespace ocs
