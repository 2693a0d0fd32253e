// GEMM kernels: C[M,N] = A[M,K] * B[N,K]^T, both operands K-contiguous.
//
//  * half / bfloat16: LDS-staged tiles feeding v_mfma_f32_32x32x16 (fp32
//    accumulate), 4 wavefronts of 64 lanes per workgroup, each owning a 64x64
//    sub-tile as 2x2 MFMA blocks.
//  * fp32 (the all-single-precision baseline mode): LDS-staged 64x64 tiles on
//    v_mfma_f32_32x32x2_f32.
//
// Optional bias add, fp32 accumulate-into-C, low-precision output, and a
// split-K form writing fp32 partials that a second kernel sums in a fixed
// order (deterministic).
#include "common.h"

namespace lstm {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_PAD = 8;               // 16 bytes per row: spreads 16-byte reads over the banks
constexpr int LDS_LD = BK + LDS_PAD;     // elements per LDS row
constexpr int THREADS = 256;

struct KernArgs {
    const void *A;
    const void *B;
    void *C;
    const void *bias;
    int M, N, K;
    int64_t lda, ldb, ldc;
    int out_lp, accumulate;
    float *ws;          // split-K partials or null
    int k_chunk;        // K range handled by one blockIdx.z
    int vec_ok;         // rows 16-byte aligned and K % 8 == 0: 16-byte global loads allowed
    int vec_out;        // 16-bit C with 16-byte aligned rows: 16-byte global stores allowed
    // blocked operands in the "rows are K" role only: batch of GEMMs (blockIdx.y) whose K rows are
    // interleaved in memory.  K tile t of batch entry y is block row
    //   (t / seg_len) * seg_stride + t % seg_len + y * seg_len      (seg_len = 0: plain, one GEMM)
    int seg_len, seg_stride;
    int64_t batch_c;    // elements between the results of consecutive batch entries
    // second product of the launch (segmented form only): tile columns tiles_n1 .. take B2 / C2 / N2 / ldb2 / ldc2
    const void *B2;
    void *C2;
    int N2, tiles_n1;
    int64_t ldb2, ldc2;
};

// 8 consecutive lp elements of row `row` at column k; zero outside the operand.
// VEC: aligned rows and K bounds that are multiples of 8 -> one unconditional
// 16-byte load from a clamped address, masked afterwards, so that the loads of
// a tile issue back to back.  Otherwise element-wise guarded loads.
template <typename T, bool VEC>
__device__ inline u32x4 load8(const T *base, int64_t ld, int row, int nrows, int k, int ksafe, int kend) {
    if constexpr (VEC) {
        const bool ok = row < nrows && k < kend;
        const int rr = row < nrows ? row : 0;
        const int kk = k < kend ? k : ksafe;
        u32x4 v = *reinterpret_cast<const u32x4 *>(base + (int64_t)rr * ld + kk);
        if (!ok) v = u32x4{0u, 0u, 0u, 0u};
        return v;
    } else {
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (row >= nrows || k >= kend) return v;
        const uint16_t *p = reinterpret_cast<const uint16_t *>(base + (int64_t)row * ld + k);
        uint16_t tmp[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) tmp[j] = (k + j < kend) ? p[j] : (uint16_t)0;
        v.x = tmp[0] | ((uint32_t)tmp[1] << 16);
        v.y = tmp[2] | ((uint32_t)tmp[3] << 16);
        v.z = tmp[4] | ((uint32_t)tmp[5] << 16);
        v.w = tmp[6] | ((uint32_t)tmp[7] << 16);
        return v;
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(THREADS) void gemm_nt_mfma_kernel(KernArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDS_LD];

    const T *A = reinterpret_cast<const T *>(a.A);
    const T *B = reinterpret_cast<const T *>(a.B);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // each thread moves 4 + 4 vectors of 8 elements per K tile
    u32x4 ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int v = tid + THREADS * i;
            int row = v >> 3, kv = (v & 7) * 8;
            ra[i] = load8<T, VEC>(A, a.lda, m0 + row, a.M, k0 + kv, kbeg, kend);
            rb[i] = load8<T, VEC>(B, a.ldb, n0 + row, a.N, k0 + kv, kbeg, kend);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int v = tid + THREADS * i;
            int row = v >> 3, kv = (v & 7) * 8;
            *reinterpret_cast<u32x4 *>(&As[buf][row * LDS_LD + kv]) = ra[i];
            *reinterpret_cast<u32x4 *>(&Bs[buf][row * LDS_LD + kv]) = rb[i];
        }
    };

    const int ntiles = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;
    if (ntiles > 0) {
        gload(kbeg);
        sstore(0);
    }
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) gload(kbeg + (t + 1) * BK);
        const int lrow = lane & 31, lk = (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            u32x4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = *reinterpret_cast<const u32x4 *>(&As[buf][(wm * 64 + i * 32 + lrow) * LDS_LD + ks * 16 + lk]);
                fb[i] = *reinterpret_cast<const u32x4 *>(&Bs[buf][(wn * 64 + i * 32 + lrow) * LDS_LD + ks * 16 + lk]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = Lp<T>::mfma(fa[i], fb[j], acc[i][j]);
        }
        if (t + 1 < ntiles) sstore(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, for each 32x32 block, column (lane%32) and rows
    // 8*(r/4) + 4*(lane/32) + r%4, r = 0..15
    const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
    const T *bias = reinterpret_cast<const T *>(a.bias);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + col_l;
            if (col >= a.N) continue;
            const float bv = (bias && blockIdx.z == 0) ? Lp<T>::to_f(bias[col]) : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 64 + i * 32 + (r >> 2) * 8 + rgrp + (r & 3);
                if (row >= a.M) continue;
                float v = acc[i][j][r] + bv;
                if (a.ws) {
                    a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
                } else if (a.out_lp) {
                    reinterpret_cast<T *>(a.C)[(int64_t)row * a.ldc + col] = Lp<T>::from_f(v);
                } else {
                    float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
                    *c = a.accumulate ? (*c + v) : v;
                }
            }
        }
}

// Large-tile variant for the whole-sequence GEMMs: 256x256 workgroup tile, eight
// wavefronts (two per SIMD, so one can issue MFMAs while the other waits on LDS
// or the barrier) in a 4x2 arrangement, each owning 64x128 (4x8 blocks of the
// 16x16x32 MFMA, 128 accumulator registers).  K tile 64, two LDS buffers (2 x 72 KB with
// padding) and two register sets: while tile t is multiplied out of LDS, tile
// t+1 sits in (or is arriving into) one register set and tile t+2 is in flight
// into the other, which covers the L2/HBM latency of about two tile times.
// The steady-state loop body is branch-free so that the wait before each
// register->LDS copy covers only that set's loads.
//
// Two operand layouts:
//   TRANS = false: C = A B^T with A[M,K], B[N,K], K contiguous (forward
//                  projection, data gradient).  LDS rows are operand rows; one
//                  16-byte LDS read per lane is one MFMA fragment.
//   TRANS = true : C = A^T B with A[K,M], B[K,N], M / N contiguous (weight
//                  gradients dA^T X, contraction over all T*B rows).  The tile
//                  is kept as it lies in memory ([k][m]) and the fragments are
//                  read with the LDS transpose read, which hands lane i of a
//                  16-lane group the 4 k-values of column i: no transposed copy
//                  of the activations is ever made.
// Aligned operands only (every leading dimension, and K resp. M/N, a multiple of 8).
constexpr int GBM = 256, GBN = 256, GBK = 64;
constexpr int GTHREADS = 512;
constexpr int GLD = GBK + LDS_PAD;               // row pitch, rows = operand rows
constexpr int GLDT = GBM + 16;                   // row pitch, rows = k (transposed form): 8 consecutive rows x 32 bytes cover all banks once
constexpr int GVPR = GBK / 8;                    // 16-byte vectors per operand row of a K tile
constexpr int GVPK = GBM / 8;                    // 16-byte vectors per k row (transposed form)
static_assert(GBK * GLDT <= GBM * GLD, "the transposed layout fits the buffers of the other one");

struct BigSmem {
    uint16_t a[2][GBM * GLD];
    uint16_t b[2][GBN * GLD];
};

typedef short v4s __attribute__((ext_vector_type(4)));

// Fragment of the 16x16x32 MFMA (lane = 16 * (k / 8) + row) out of a [k][m] tile: columns m0 .. m0 + 15, 32-deep step
// q, via two transpose reads: each 16-lane group reads 4 k-rows x 16 columns per instruction and every lane receives
// the 4 k-values of column (lane % 16).
// PERM (both operands of the product are read this way): k-group g of the MFMA takes tile rows 4 g .. 4 g + 3 and
// 16 + 4 g .. 16 + 4 g + 3 of the step instead of 8 g .. 8 g + 7 (any assignment of tile rows to the MFMA's
// contraction slots is right as long as both operands use it), so that one instruction touches 16 consecutive rows.
template <bool PERM>
__device__ __forceinline__ u32x4 read_frag_tr16(const uint16_t *tile, int m0, int q, int lane) {
    const int g = lane >> 4, i = lane & 15;
    const uint16_t *p = tile + (q * 32 + (PERM ? 4 : 8) * g + (i >> 2)) * GLDT + m0 + 4 * (i & 3);
    typedef __attribute__((address_space(3))) v4s *lds_v4s;
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + (PERM ? 16 : 4) * GLDT));
    struct { v4s l, h; } both = {lo, hi};
    return __builtin_bit_cast(u32x4, both);
}

// Result tile of the large-tile kernel: bias, then split-K partials, 16-bit or fp32 result.  Accumulator block
// (i, j) of a wavefront's 64 x 128 holds rows 16 i + 4 (lane / 16) + r, column 16 j + lane % 16.
template <typename T, int GTHREADS>
__device__ __forceinline__ void big_epilogue16(const KernArgs &a, BigSmem &sm, v4f (&acc)[4][8], int m0, int n0, int wm, int wn,
                                               int lane, int tid) {
    const int col_l = lane & 15, rgrp = (lane >> 4) * 4;
    const T *bias = reinterpret_cast<const T *>(a.bias);
    if (a.out_lp && !a.ws && a.vec_out) {
        // 16-bit result: the accumulators hold one column per lane, which would go out as 2-byte
        // stores.  Stage the tile in LDS (free once the last K tile has been multiplied) and
        // write it as whole 512-byte row segments instead.
        constexpr int OLD = GBN + 8;                       // staging row pitch (elements)
        static_assert(GBM * OLD * 2 <= (int)sizeof(BigSmem), "staged tile must fit the operand buffers");
        T *stage = reinterpret_cast<T *>(&sm);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cl = wn * 128 + j * 16 + col_l;
            const int col = n0 + cl;
            const float bv = (bias && col < a.N) ? Lp<T>::to_f(bias[col]) : 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) stage[(wm * 64 + i * 16 + rgrp + r) * OLD + cl] = Lp<T>::from_f(acc[i][j][r] + bv);
        }
        __syncthreads();
        T *C = reinterpret_cast<T *>(a.C);
#pragma unroll 4
        for (int v = tid; v < GBM * (GBN / 8); v += GTHREADS) {
            const int rl = v / (GBN / 8), cl = (v % (GBN / 8)) * 8;
            const int row = m0 + rl, col = n0 + cl;
            if (row >= a.M || col >= a.N) continue;
            const u32x4 val = *reinterpret_cast<const u32x4 *>(&stage[rl * OLD + cl]);
            if (col + 8 <= a.N) {
                *reinterpret_cast<u32x4 *>(&C[(int64_t)row * a.ldc + col]) = val;
            } else {
                T e[8];
                __builtin_memcpy(e, &val, 16);
                for (int q = 0; q < a.N - col; ++q) C[(int64_t)row * a.ldc + col + q] = e[q];
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int col = n0 + wn * 128 + j * 16 + col_l;
        if (col >= a.N) continue;
        const float bv = (bias && blockIdx.z == 0) ? Lp<T>::to_f(bias[col]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = m0 + wm * 64 + i * 16 + rgrp + r;
                if (row >= a.M) continue;
                const float v = acc[i][j][r] + bv;
                if (a.ws) {
                    a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
                } else if (a.out_lp) {
                    reinterpret_cast<T *>(a.C)[(int64_t)row * a.ldc + col] = Lp<T>::from_f(v);
                } else {
                    float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
                    *c = a.accumulate ? (*c + v) : v;
                }
            }
    }
}

// TA / TB_: operand A / B is in the transposed role (its rows are the contraction index).
// BLK: operands are stored in 64x64 blocks ([row block][column block][64][64], zero padded to
//      whole blocks; lda / ldb then hold the number of column blocks per row block and K is a
//      multiple of 64).  A K tile of an operand is then four contiguous 8 KB blocks instead of 256
//      row segments of 128 bytes, which is what the L2 -> CU path streams at full rate.
// PP:  steady state in the ping-pong slot schedule (below) instead of the plain two-stage loop.
// SEG: a batch of products (blockIdx.y) whose K rows interleave in memory (see KernArgs::seg_len).
template <typename T, bool TA, bool TB_, bool BLK, bool PP, bool SEG = false>
__global__ __launch_bounds__(GTHREADS) void gemm_mfma_big_kernel(KernArgs a_in, int tiles_m, int tiles_n) {
    constexpr int GNV = GBM * GBK / 8 / GTHREADS;  // 16-byte vectors per thread, operand and K tile (4)
    __shared__ __attribute__((aligned(16))) BigSmem sm;
    KernArgs a = a_in;
    const T *A = reinterpret_cast<const T *>(a.A);
    const T *B = reinterpret_cast<const T *>(a.B);
    int bx = blockIdx.x;
    if constexpr (SEG) {
        // batch entry y: its K rows start seg_len block rows further on in both operands.  The tiles of one
        // entry all stream the same B panel, so they should share an L2: workgroup id -> (XCD = id % 8, slot =
        // id / 8), and an XCD's slots walk the tiles of the entries 8 k + XCD one entry after the other (plain
        // (x, y) order puts the tiles of an entry on neighbouring XCDs and every one of them fetches the panel).
        static_assert(!SEG || (BLK && TA && TB_), "segmented K only for blocked operands in the rows-are-K role");
        int64_t y = blockIdx.y;
        if (gridDim.y % 8 == 0) {
            const int id = (int)blockIdx.y * (int)gridDim.x + (int)blockIdx.x, slot = id >> 3;
            bx = slot % (int)gridDim.x;
            y = (int64_t)(slot / (int)gridDim.x) * 8 + (id & 7);
        }
        A += y * a.seg_len * a.lda * 4096;
        if (a.B2) {
            // two products share the launch: which one this tile column belongs to (same order as below: the tiles of
            // an entry are walked tile column by tile column)
            const int bh_ = min(8, tiles_m);
            const int tn_ = (bx % (8 * tiles_n)) / bh_;
            if (tn_ >= a.tiles_n1) {
                B = reinterpret_cast<const T *>(a.B2);
                a.C = a.C2; a.N = a.N2; a.ldb = a.ldb2; a.ldc = a.ldc2;
            }
        }
        B += y * a.seg_len * a.ldb * 4096;
        a.C = reinterpret_cast<char *>(a.C) + y * a.batch_c * (a.out_lp ? (int64_t)sizeof(T) : 4);
    }
    // K tile -> block row of a "rows are K" blocked operand
    auto krow = [&](int tile) -> uint32_t {
        if constexpr (SEG) return (uint32_t)((tile / a.seg_len) * a.seg_stride + tile % a.seg_len);
        return (uint32_t)tile;
    };
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;       // 4 x 2 wavefronts of 64 x 128
    // tile order: workgroups of one XCD (id % 8) take neighbouring tiles, and tiles
    // are walked in bands of 8 tile rows so that a band's A and B panels stay in L2
    const int total = tiles_m * tiles_n;
    int lin = bx;
    if (!SEG && total % 8 == 0) lin = (lin % 8) * (total / 8) + lin / 8;
    const int band = 8 * tiles_n;
    const int b0 = (lin / band) * 8;
    const int bh = min(8, tiles_m - b0);
    const int tm = b0 + (lin % band) % bh;
    int tn = (lin % band) / bh;
    if constexpr (SEG) {
        if (a.B2 && tn >= a.tiles_n1) tn -= a.tiles_n1;   // (operands switched above)
    }
    const int m0 = tm * GBM, n0 = tn * GBN;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);

    // 16x16x32 MFMAs: block (i, j) of the wavefront's 64 x 128.  Per flop this form moves half as many accumulator
    // registers as the 32x32x16 one, and on real (non-constant) operands, where the clock is set by the power cap,
    // that is worth more than anything the schedule can win (register-resident loops: 2.03 against 1.70 PFLOP/s).
    v4f acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

    // Per-thread element offsets of the vectors this thread copies for K tile 0 (32-bit: the
    // host checks that both operands span less than 2^31 elements) and the step to the next
    // tile.  Rows / columns / blocks outside the operand are clamped to the first one: what
    // they contribute only reaches accumulator rows/columns that are never stored.
    uint32_t oa[GNV], ob[GNV];
    uint32_t step_a, step_b;
    auto setup = [&](bool trans, int x0, int extent, int64_t ld, uint32_t (&o)[GNV], uint32_t &step) {
#pragma unroll
        for (int i = 0; i < GNV; ++i) {
            const int v = tid + GTHREADS * i;
            if constexpr (BLK) {
                // the tile is four 64x64 blocks of 512 vectors each
                const int xb = x0 / 64 + v / 512, nxb = (extent + 63) / 64;
                const int xbc = xb < nxb ? xb : 0;
                const int ncb = (int)ld;
                // block offset only (the same for the whole workgroup: it stays in scalar registers); the thread's
                // vector inside the block, tid * 8 elements, is added at the access
                static_assert(!BLK || GTHREADS == 512, "vector v % 512 of a block is the thread's own");
                o[i] = (uint32_t)__builtin_amdgcn_readfirstlane(trans ? ((kbeg / 64) * ncb + xbc) * 4096 : (xbc * ncb + kbeg / 64) * 4096);
            } else if (trans) {
                const int krow = v / GVPK, xv = (v % GVPK) * 8;
                o[i] = (uint32_t)((kbeg + krow) * ld + (x0 + xv < extent ? x0 + xv : 0));
            } else {
                const int row = v / GVPR, kv = (v % GVPR) * 8;
                o[i] = (uint32_t)((x0 + row < extent ? x0 + row : 0) * ld + kv + kbeg);
            }
        }
        if constexpr (BLK) step = trans ? (uint32_t)ld * 4096u : 4096u;
        else step = trans ? (uint32_t)(GBK * ld) : (uint32_t)GBK;
    };
    setup(TA, m0, a.M, a.lda, oa, step_a);
    setup(TB_, n0, a.N, a.ldb, ob, step_b);
    const int klen = kend > kbeg ? kend - kbeg : 0;
    const int ntiles = (klen + GBK - 1) / GBK;
    const int nfull = klen / GBK;                  // tiles that lie wholly inside the K range

    const uint32_t lane_el = BLK ? (uint32_t)tid * 8u : 0u;
    auto src_a = [&](int i, uint32_t add) { return reinterpret_cast<const u32x4 *>(A + (oa[i] + add) + lane_el); };
    auto src_b = [&](int i, uint32_t add) { return reinterpret_cast<const u32x4 *>(B + (ob[i] + add) + lane_el); };
    u32x4 a0[GNV], b0r[GNV], a1[GNV], b1r[GNV];    // register set 0 and 1
    auto gload_full = [&](u32x4 (&ra)[GNV], u32x4 (&rb)[GNV], int tile) {
#pragma unroll
        for (int i = 0; i < GNV; ++i) {
            ra[i] = *src_a(i, (TA ? krow(tile) : (uint32_t)tile) * step_a);
            rb[i] = *src_b(i, (TB_ ? krow(tile) : (uint32_t)tile) * step_b);
        }
    };
    auto gload_any = [&](u32x4 (&ra)[GNV], u32x4 (&rb)[GNV], int tile) {   // also the last, partial tile
#pragma unroll
        for (int i = 0; i < GNV; ++i) {
            const int v = tid + GTHREADS * i;
            // first k of this vector inside the tile (blocked operands are padded: always inside)
            const int ka = BLK ? 0 : (TA ? v / GVPK : (v % GVPR) * 8);
            const int kb = BLK ? 0 : (TB_ ? v / GVPK : (v % GVPR) * 8);
            ra[i] = tile * GBK + ka < klen ? *src_a(i, (TA ? krow(tile) : (uint32_t)tile) * step_a)
                                           : u32x4{0u, 0u, 0u, 0u};
            rb[i] = tile * GBK + kb < klen ? *src_b(i, (TB_ ? krow(tile) : (uint32_t)tile) * step_b)
                                           : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto lds_off = [&](bool trans, int i) {
        const int v = tid + GTHREADS * i;
        if constexpr (BLK) {
            const int blk = v / 512, w = v % 512;
            return trans ? (w >> 3) * GLDT + blk * 64 + (w & 7) * 8 : (blk * 64 + (w >> 3)) * GLD + (w & 7) * 8;
        }
        else return trans ? (v / GVPK) * GLDT + (v % GVPK) * 8 : (v / GVPR) * GLD + (v % GVPR) * 8;
    };
    auto sstore = [&](const u32x4 (&ra)[GNV], const u32x4 (&rb)[GNV], int buf) {
#pragma unroll
        for (int i = 0; i < GNV; ++i) {
            *reinterpret_cast<u32x4 *>(&sm.a[buf][lds_off(TA, i)]) = ra[i];
            *reinterpret_cast<u32x4 *>(&sm.b[buf][lds_off(TB_, i)]) = rb[i];
        }
    };
    const int lrow = lane & 15, lk = (lane >> 4) * 8;
    // fragments of 32-deep step q: A rows (wm 64 + 16 i ..), B rows (wn 128 + 16 j ..)
    auto frag_a = [&](int buf, int i, int q) -> u32x4 {
        if constexpr (TA) return read_frag_tr16<TA && TB_>(sm.a[buf], wm * 64 + i * 16, q, lane);
        else return *reinterpret_cast<const u32x4 *>(&sm.a[buf][(wm * 64 + i * 16 + lrow) * GLD + lk + q * 32]);
    };
    auto frag_b = [&](int buf, int j, int q) -> u32x4 {
        if constexpr (TB_) return read_frag_tr16<TA && TB_>(sm.b[buf], wn * 128 + j * 16, q, lane);
        else return *reinterpret_cast<const u32x4 *>(&sm.b[buf][(wn * 128 + j * 16 + lrow) * GLD + lk + q * 32]);
    };
    // half steps [h0, h1) of the tile in LDS buffer `buf`: half step h = 32-deep step h / 2, column blocks 4 (h % 2) ..
    auto compute = [&](int buf, int h0, int h1) {
        u32x4 fa[4];
#pragma unroll
        for (int h = h0; h < h1; ++h) {
            const int q = h >> 1, nh = h & 1;
            u32x4 fb[4];
            if (nh == 0 || h == h0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) fa[i] = frag_a(buf, i, q);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) fb[j] = frag_b(buf, nh * 4 + j, q);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][nh * 4 + j] = Lp<T>::mfma16(fa[i], fb[j], acc[i][nh * 4 + j]);
        }
    };
    constexpr int KS = GBK / 16;                  // half steps per tile (16 MFMAs per wavefront each)

    if (ntiles > 0) {
        // prologue: tile 0 -> LDS buffer 0, tile 1 -> set 1, tile 2 -> set 0
        gload_any(a0, b0r, 0);
        if (ntiles > 1) gload_any(a1, b1r, 1);
        sstore(a0, b0r, 0);
        if (ntiles > 2) gload_any(a0, b0r, 2);
        __syncthreads();
        int t = 0;
        if constexpr (PP) {
            // Ping-pong schedule.  The first four wavefronts sit on the four SIMDs, the second four
            // share them.  Every k-step is split into a slot that reads its fragments from LDS (and
            // moves a quarter of the next tile: registers -> LDS, global -> registers) and a slot
            // that issues its MFMAs, with a workgroup barrier after every slot.  The second group
            // runs one slot behind the first, so while one wavefront of a SIMD keeps the matrix
            // pipe busy the other one uses the LDS, instead of all eight doing the same thing at
            // the same time.  Buffer safety: a tile's last fragment read (second group, k-step 3)
            // lies one slot before the first store into that buffer, its first read one slot
            // after the last store, and there is a barrier between any two slots.
            const int grp = wave >> 2;
            auto slot_barrier = [&]() {
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            };
            auto pp_tile = [&](int buf, u32x4 (&ra)[GNV], u32x4 (&rb)[GNV], int tile_next) {
                const uint32_t next_a = (TA ? krow(tile_next) : (uint32_t)tile_next) * step_a;
                const uint32_t next_b = (TB_ ? krow(tile_next) : (uint32_t)tile_next) * step_b;
                u32x4 fa[4];
#pragma unroll
                for (int ks = 0; ks < GBK / 16; ++ks) {
                    const int q = ks >> 1, nh = ks & 1;
                    u32x4 fb[4];
                    if (nh == 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) fa[i] = frag_a(buf, i, q);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) fb[j] = frag_b(buf, nh * 4 + j, q);
                    *reinterpret_cast<u32x4 *>(&sm.a[buf ^ 1][lds_off(TA, ks)]) = ra[ks];
                    *reinterpret_cast<u32x4 *>(&sm.b[buf ^ 1][lds_off(TB_, ks)]) = rb[ks];
                    ra[ks] = *src_a(ks, next_a);
                    rb[ks] = *src_b(ks, next_b);
                    slot_barrier();
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[i][nh * 4 + j] = Lp<T>::mfma16(fa[i], fb[j], acc[i][nh * 4 + j]);
                    slot_barrier();
                }
            };
            static_assert(GNV == GBK / 16, "one A and one B vector per thread and k-step");
            if (t + 4 < nfull) {
                if (grp == 1) slot_barrier();
                for (; t + 4 < nfull; t += 2) {
                    pp_tile(0, a1, b1r, t + 3);     // multiply tile t, move tile t+1, fetch tile t+3
                    pp_tile(1, a0, b0r, t + 4);     // multiply tile t+1, move tile t+2, fetch tile t+4
                }
                if (grp == 0) slot_barrier();
            }
        }
        // steady state: tiles t+3 and t+4 are full tiles, no branches in the body.  The copy of
        // the next tile into the other LDS buffer sits between the two halves of the MFMA work so
        // that it overlaps with them instead of delaying the barrier.
        for (; t + 4 < nfull; t += 2) {
            compute(0, 0, KS / 2);      // tile t
            sstore(a1, b1r, 1);         // tile t+1
            gload_full(a1, b1r, t + 3);
            compute(0, KS / 2, KS);
            __syncthreads();
            compute(1, 0, KS / 2);      // tile t+1
            sstore(a0, b0r, 0);         // tile t+2
            gload_full(a0, b0r, t + 4);
            compute(1, KS / 2, KS);
            __syncthreads();
        }
        // drain: same schedule with range checks
        for (; t < ntiles; t += 2) {
            compute(0, 0, KS);
            if (t + 1 < ntiles) sstore(a1, b1r, 1);
            if (t + 3 < ntiles) gload_any(a1, b1r, t + 3);
            __syncthreads();
            if (t + 1 < ntiles) {
                compute(1, 0, KS);
                if (t + 2 < ntiles) sstore(a0, b0r, 0);
                if (t + 4 < ntiles) gload_any(a0, b0r, t + 4);
                __syncthreads();
            }
        }
    }

    big_epilogue16<T, GTHREADS>(a, sm, acc, m0, n0, wm, wn, lane, tid);
}

// row-major [R, C] (leading dimension ld) -> 64x64 blocks, zero padded
template <typename U>
__global__ __launch_bounds__(256) void pack_blocked_kernel(const U *src, int64_t ld, int R, int C, U *dst, int ncb) {
    const int rb = blockIdx.y, cb = blockIdx.x;
    U *d = dst + ((int64_t)rb * ncb + cb) * 4096;
    for (int v = threadIdx.x; v < 4096; v += 256) {
        const int r = rb * 64 + (v >> 6), c = cb * 64 + (v & 63);
        d[v] = (r < R && c < C) ? src[(int64_t)r * ld + c] : (U)0;
    }
}

// the same for 16-bit elements in 16-byte pieces (rows 16-byte aligned, C a multiple of 8): two pieces per thread
__global__ __launch_bounds__(256) void pack_blocked_vec_kernel(const uint16_t *src, int64_t ld, int R, int C, uint16_t *dst, int ncb) {
    const int rb = blockIdx.y, cb = blockIdx.x;
    u32x4 *d = reinterpret_cast<u32x4 *>(dst + ((int64_t)rb * ncb + cb) * 4096);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int v = threadIdx.x + 256 * i;
        const int r = rb * 64 + (v >> 3), c = cb * 64 + (v & 7) * 8;
        d[v] = (r < R && c < C) ? *reinterpret_cast<const u32x4 *>(src + (int64_t)r * ld + c) : u32x4{0u, 0u, 0u, 0u};
    }
}

// fp32 baseline-mode GEMM: 64x64 tile, 32-deep K slices, four wavefronts with one 32x32 block each on
// v_mfma_f32_32x32x2_f32 (fp32 products, fp32 accumulate).  That instruction takes k = 0 from lanes
// 0..31 and k = 1 from lanes 32..63; the order of k inside a slice is free as long as both operands
// agree, so lane half q contracts k = 16 q + j in MFMA j and a lane's operands are 16 consecutive
// floats of its row (four 16-byte LDS reads per operand and slice).
constexpr int SBM = 64, SBN = 64, SBK = 32;
constexpr int SLD = SBK + 4;             // floats per LDS row: 16-byte reads of 8 rows cover all banks

// 4 consecutive floats of row `row` at column k; zero outside the operand
template <bool VEC>
__device__ inline v4f load4(const float *base, int64_t ld, int row, int nrows, int k, int ksafe, int kend) {
    if constexpr (VEC) {
        const bool ok = row < nrows && k < kend;
        const int rr = row < nrows ? row : 0;
        const int kk = k < kend ? k : ksafe;
        v4f v = *reinterpret_cast<const v4f *>(base + (int64_t)rr * ld + kk);
        if (!ok) v = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        return v;
    } else {
        v4f v = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        if (row >= nrows) return v;
        const float *p = base + (int64_t)row * ld + k;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (k + j < kend) v[j] = p[j];
        return v;
    }
}

template <bool VEC>
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(KernArgs a) {
    __shared__ __attribute__((aligned(16))) float As[2][SBM * SLD];
    __shared__ __attribute__((aligned(16))) float Bs[2][SBN * SLD];
    const float *A = reinterpret_cast<const float *>(a.A);
    const float *B = reinterpret_cast<const float *>(a.B);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * SBM, n0 = blockIdx.x * SBN;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);

    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    // each thread moves 2 + 2 vectors of 4 floats per K slice
    v4f ra[2], rb[2];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int v = tid + 256 * i;
            const int row = v >> 3, kv = (v & 7) * 4;
            ra[i] = load4<VEC>(A, a.lda, m0 + row, a.M, k0 + kv, kbeg, kend);
            rb[i] = load4<VEC>(B, a.ldb, n0 + row, a.N, k0 + kv, kbeg, kend);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int v = tid + 256 * i;
            const int row = v >> 3, kv = (v & 7) * 4;
            *reinterpret_cast<v4f *>(&As[buf][row * SLD + kv]) = ra[i];
            *reinterpret_cast<v4f *>(&Bs[buf][row * SLD + kv]) = rb[i];
        }
    };

    const int ntiles = (kend > kbeg) ? (kend - kbeg + SBK - 1) / SBK : 0;
    if (ntiles > 0) {
        gload(kbeg);
        sstore(0);
    }
    __syncthreads();
    const int lrow = lane & 31, lk = (lane >> 5) * 16;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) gload(kbeg + (t + 1) * SBK);
        v4f fa[4], fb[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            fa[q] = *reinterpret_cast<const v4f *>(&As[buf][(wm * 32 + lrow) * SLD + lk + q * 4]);
            fb[q] = *reinterpret_cast<const v4f *>(&Bs[buf][(wn * 32 + lrow) * SLD + lk + q * 4]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[q][j], fb[q][j], acc, 0, 0, 0);
        if (t + 1 < ntiles) sstore(buf ^ 1);
        __syncthreads();
    }

    // lane holds column lane % 32 and rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15, of its block
    const float *bias = reinterpret_cast<const float *>(a.bias);
    const int col = n0 + wn * 32 + lrow;
    if (col >= a.N) return;
    const float bv = (bias && blockIdx.z == 0) ? bias[col] : 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row >= a.M) continue;
        const float v = acc[r] + bv;
        if (a.ws) {
            a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
        } else {
            float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
            *c = a.accumulate ? (*c + v) : v;
        }
    }
}

// The same contraction for results of few tiles (the per-time-step products of the fp32 mode): a
// 32x32 tile per workgroup and 128-deep K slices (few workgroups, so what a launch costs is the
// chain of load latencies: four vectors per thread and operand are in flight at a time); the four
// wavefronts each contract a quarter of every slice (k = 32 w + 16 q + j for wavefront w, lane
// half q, MFMA j) and their partial blocks are added through LDS.
constexpr int SSK = 128, SSLD = SSK + 4;
template <bool VEC>
__global__ __launch_bounds__(256) void gemm_nt_f32_small_kernel(KernArgs a) {
    __shared__ __attribute__((aligned(16))) float As[2][32 * SSLD];
    __shared__ __attribute__((aligned(16))) float Bs[2][32 * SSLD];
    __shared__ float red[4][16 * 64];
    const float *A = reinterpret_cast<const float *>(a.A);
    const float *B = reinterpret_cast<const float *>(a.B);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);

    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    v4f ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + 256 * i;
            const int row = v >> 5, kv = (v & 31) * 4;
            ra[i] = load4<VEC>(A, a.lda, m0 + row, a.M, k0 + kv, kbeg, kend);
            rb[i] = load4<VEC>(B, a.ldb, n0 + row, a.N, k0 + kv, kbeg, kend);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = tid + 256 * i;
            const int row = v >> 5, kv = (v & 31) * 4;
            *reinterpret_cast<v4f *>(&As[buf][row * SSLD + kv]) = ra[i];
            *reinterpret_cast<v4f *>(&Bs[buf][row * SSLD + kv]) = rb[i];
        }
    };

    const int ntiles = (kend > kbeg) ? (kend - kbeg + SSK - 1) / SSK : 0;
    if (ntiles > 0) {
        gload(kbeg);
        sstore(0);
    }
    __syncthreads();
    const int lrow = lane & 31, lk = wave * 32 + (lane >> 5) * 16;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) gload(kbeg + (t + 1) * SSK);
        v4f fa[4], fb[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            fa[q] = *reinterpret_cast<const v4f *>(&As[buf][lrow * SSLD + lk + q * 4]);
            fb[q] = *reinterpret_cast<const v4f *>(&Bs[buf][lrow * SSLD + lk + q * 4]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[q][j], fb[q][j], acc, 0, 0, 0);
        if (t + 1 < ntiles) sstore(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][r * 64 + lane] = acc[r];
    __syncthreads();

    // element (r, l) of a block: column l % 32, row 8*(r/4) + 4*(l/32) + r%4
    const float *bias = reinterpret_cast<const float *>(a.bias);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i;
        const int r = e >> 6, l = e & 63;
        const int row = m0 + (r >> 2) * 8 + (l >> 5) * 4 + (r & 3), col = n0 + (l & 31);
        if (row >= a.M || col >= a.N) continue;
        float v = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
        if (bias && blockIdx.z == 0) v += bias[col];
        if (a.ws) {
            a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
        } else {
            float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
            *c = a.accumulate ? (*c + v) : v;
        }
    }
}

// sum split-K partials in index order and store
template <typename T>
__global__ void splitk_reduce_kernel(const float *ws, int splits, int M, int N, void *C, int64_t ldc, int out_lp,
                                     int accumulate) {
    const int64_t total = (int64_t)M * N;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int z = 0; z < splits; ++z) s += ws[(int64_t)z * total + e];
        const int row = (int)(e / N), col = (int)(e % N);
        if (out_lp) {
            reinterpret_cast<T *>(C)[(int64_t)row * ldc + col] = Lp<T>::from_f(s);
        } else {
            float *c = reinterpret_cast<float *>(C) + (int64_t)row * ldc + col;
            *c = accumulate ? (*c + s) : s;
        }
    }
}

inline bool use_big_tiles(int dtype, int M, int N) { return dtype != LSTM_DTYPE_FP32 && M >= 192 && N >= 192; }
inline bool fits_32bit(int64_t rows_a, int64_t lda, int64_t rows_b, int64_t ldb) {
    return rows_a * lda < (int64_t)1 << 31 && rows_b * ldb < (int64_t)1 << 31;
}

template <typename T>
int finish_splitk(const GemmArgs &g, int splits, hipStream_t stream) {
    if (splits <= 1) return LSTM_OK;
    const int64_t total = (int64_t)g.M * g.N;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(splitk_reduce_kernel<T>, dim3(blocks), dim3(256), 0, stream, g.splitk_ws, splits, g.M, g.N, g.C,
                       g.ldc, g.out_lp, g.accumulate);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace
// 16-bit C = sum of `splits` fp32 partial results [split][M][N], added up in index order
int splitk_reduce(int dtype, const float *ws, int splits, int M, int N, void *C, int64_t ldc, hipStream_t stream) {
    GemmArgs g{};
    g.splitk_ws = const_cast<float *>(ws); g.M = M; g.N = N; g.C = C; g.ldc = ldc; g.out_lp = 1;
    if (dtype == LSTM_DTYPE_FP16) return finish_splitk<_Float16>(g, splits, stream);
    if (dtype == LSTM_DTYPE_BF16) return finish_splitk<bf16_t>(g, splits, stream);
    set_error("splitk_reduce: 16-bit types only");
    return LSTM_ERR_UNSUPPORTED;
}
namespace {
// Bytes a GEMM moves if every operand is read once and the result written once
// (read too when accumulating): what the event timer accounts the launch with.
template <typename T, typename Args>
static double gemm_algorithmic_bytes(const Args &g) {
    const double out = (double)g.M * g.N * (g.out_lp ? sizeof(T) : 4.0);
    return ((double)g.M + g.N) * g.K * sizeof(T) + out * (g.accumulate ? 2.0 : 1.0);
}

template <typename T>
int launch(const GemmArgs &g, hipStream_t stream) {
    constexpr bool is_f32 = sizeof(T) == 4;
    constexpr int vec = 16 / (int)sizeof(T);     // elements per 16-byte load
    const bool aligned = g.K % vec == 0 && g.lda % vec == 0 && g.ldb % vec == 0 && ((uintptr_t)g.A % 16 == 0) &&
                         ((uintptr_t)g.B % 16 == 0);
    const bool big = !is_f32 && aligned && fits_32bit(g.M, g.lda, g.N, g.ldb) &&
                     use_big_tiles(is_f32 ? LSTM_DTYPE_FP32 : LSTM_DTYPE_FP16, g.M, g.N);
    // fp32: 32x32 tiles while 64x64 ones would leave compute units without a workgroup
    const int asked = (g.splitk_ws && g.splits > 1) ? g.splits : 1;
    const bool small32 = is_f32 && (int64_t)((g.M + SBM - 1) / SBM) * ((g.N + SBN - 1) / SBN) * asked < 256;
    const int bm = is_f32 ? (small32 ? 32 : SBM) : (big ? GBM : BM), bn = is_f32 ? (small32 ? 32 : SBN) : (big ? GBN : BN);
    const int bk = is_f32 ? SBK : BK;
    KernArgs a{};
    a.A = g.A; a.B = g.B; a.C = g.C; a.bias = g.bias;
    a.M = g.M; a.N = g.N; a.K = g.K;
    a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
    a.out_lp = g.out_lp; a.accumulate = g.accumulate;
    int splits = (g.splitk_ws && g.splits > 1) ? g.splits : 1;
    int k_chunk = g.K;
    if (splits > 1) {
        k_chunk = ((g.K + splits - 1) / splits + bk - 1) / bk * bk;
        splits = (g.K + k_chunk - 1) / k_chunk;
    }
    a.ws = splits > 1 ? g.splitk_ws : nullptr;
    a.k_chunk = k_chunk;
    a.vec_ok = aligned ? 1 : 0;
    a.vec_out = (g.out_lp && g.ldc % 8 == 0 && (uintptr_t)g.C % 16 == 0) ? 1 : 0;
    const int tiles_m = (g.M + bm - 1) / bm, tiles_n = (g.N + bn - 1) / bn;
    if (tiles_m > 65535 || splits > 65535 || (int64_t)tiles_m * tiles_n > 0x7fffffff) {
        set_error("gemm_nt: grid too large (M=%d N=%d splits=%d)", g.M, g.N, splits);
        return LSTM_ERR_UNSUPPORTED;
    }
    KernelTimer timer(g.kclass, stream, 2.0 * g.M * g.N * g.K, gemm_algorithmic_bytes<T>(g));
    if constexpr (is_f32) {
        if (small32 && a.vec_ok) {
            hipLaunchKernelGGL(gemm_nt_f32_small_kernel<true>, dim3(tiles_n, tiles_m, splits), dim3(256), 0, stream, a);
        } else if (small32) {
            hipLaunchKernelGGL(gemm_nt_f32_small_kernel<false>, dim3(tiles_n, tiles_m, splits), dim3(256), 0, stream, a);
        } else if (a.vec_ok) {
            hipLaunchKernelGGL(gemm_nt_f32_kernel<true>, dim3(tiles_n, tiles_m, splits), dim3(256), 0, stream, a);
        } else {
            hipLaunchKernelGGL(gemm_nt_f32_kernel<false>, dim3(tiles_n, tiles_m, splits), dim3(256), 0, stream, a);
        }
    } else {
        if (big) {
            hipLaunchKernelGGL((gemm_mfma_big_kernel<T, false, false, false, false>), dim3(tiles_m * tiles_n, 1, splits), dim3(GTHREADS), 0,
                               stream, a, tiles_m, tiles_n);
        } else if (a.vec_ok) {
            hipLaunchKernelGGL((gemm_nt_mfma_kernel<T, true>), dim3(tiles_n, tiles_m, splits), dim3(THREADS), 0, stream, a);
        } else {
            hipLaunchKernelGGL((gemm_nt_mfma_kernel<T, false>), dim3(tiles_n, tiles_m, splits), dim3(THREADS), 0, stream, a);
        }
    }
    LSTM_LAUNCH_CHECK();
    return finish_splitk<T>(g, splits, stream);
}

// C[M,N] = A^T B with A[K,M] (lda), B[K,N] (ldb); only the large-tile kernel implements it
template <typename T>
int launch_tn(const GemmArgs &g, hipStream_t stream) {
    KernArgs a{};
    a.A = g.A; a.B = g.B; a.C = g.C; a.bias = nullptr;
    a.M = g.M; a.N = g.N; a.K = g.K;
    a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
    a.out_lp = g.out_lp; a.accumulate = g.accumulate;
    int splits = (g.splitk_ws && g.splits > 1) ? g.splits : 1;
    int k_chunk = g.K;
    if (splits > 1) {
        k_chunk = ((g.K + splits - 1) / splits + GBK - 1) / GBK * GBK;
        splits = (g.K + k_chunk - 1) / k_chunk;
    }
    a.ws = splits > 1 ? g.splitk_ws : nullptr;
    a.k_chunk = k_chunk;
    a.vec_ok = 1;
    a.vec_out = (g.out_lp && g.ldc % 8 == 0 && (uintptr_t)g.C % 16 == 0) ? 1 : 0;
    const int tiles_m = (g.M + GBM - 1) / GBM, tiles_n = (g.N + GBN - 1) / GBN;
    KernelTimer timer(g.kclass, stream, 2.0 * g.M * g.N * g.K, gemm_algorithmic_bytes<T>(g));
    hipLaunchKernelGGL((gemm_mfma_big_kernel<T, true, true, false, false>), dim3(tiles_m * tiles_n, 1, splits), dim3(GTHREADS), 0, stream,
                       a, tiles_m, tiles_n);
    LSTM_LAUNCH_CHECK();
    return finish_splitk<T>(g, splits, stream);
}

}  // namespace

int gemm_pick_splits(int dtype, int M, int N, int K) {
    // enough workgroups to cover the 256 compute units, each with a K range worth pipelining
    const bool big = use_big_tiles(dtype, M, N);
    const int bm = big ? GBM : BM, bn = big ? GBN : BN;
    const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const long enough = big ? 256 : 512;
    if (tiles >= enough || K < 8 * BK) return 1;
    long want = (enough + tiles - 1) / tiles;
    long maxs = K / (4 * BK);
    if (want > maxs) want = maxs;
    if (want > 256) want = 256;
    // every split writes an fp32 copy of the result that the reduction reads back: keep that traffic
    // (it, not the products, is what a small-output contraction costs) within a few megabytes
    // ... but no split longer than 32 K tiles while workgroups are still to be had
    long cap = (8L << 20) / ((long)M * N * 4);
    const long by_length = (K + 32 * BK - 1) / (32 * BK);
    if (cap < by_length) cap = by_length;
    if (want > cap) want = cap;
    return want < 1 ? 1 : (int)want;
}

int gemm_nt(int dtype, const GemmArgs &g, hipStream_t stream) {
    if (g.M <= 0 || g.N <= 0) return LSTM_OK;
    if (!g.A || !g.B || !g.C || g.K < 0) {
        set_error("gemm_nt: null operand");
        return LSTM_ERR_INVALID;
    }
    switch (dtype) {
        case LSTM_DTYPE_FP32: return launch<float>(g, stream);
        case LSTM_DTYPE_FP16: return launch<_Float16>(g, stream);
        case LSTM_DTYPE_BF16: return launch<bf16_t>(g, stream);
    }
    set_error("gemm_nt: bad dtype %d", dtype);
    return LSTM_ERR_INVALID;
}

namespace {
template <typename T>
int launch_blocked(const BlockedGemmArgs &g, hipStream_t stream) {
    KernArgs a{};
    a.A = g.A.ptr; a.B = g.B.ptr; a.C = g.C; a.bias = g.bias;
    a.M = g.M; a.N = g.N;
    a.K = (g.K + 63) / 64 * 64;                  // operands are zero padded to whole blocks
    a.lda = g.A.ncb; a.ldb = g.B.ncb; a.ldc = g.ldc;
    a.out_lp = g.out_lp; a.accumulate = g.accumulate;
    int splits = (g.splitk_ws && g.splits > 1) ? g.splits : 1;
    int k_chunk = a.K;
    if (splits > 1) {
        k_chunk = ((a.K + splits - 1) / splits + GBK - 1) / GBK * GBK;
        splits = (a.K + k_chunk - 1) / k_chunk;
    }
    a.ws = splits > 1 ? g.splitk_ws : nullptr;
    a.k_chunk = k_chunk;
    a.vec_ok = 1;
    a.vec_out = (g.out_lp && g.ldc % 8 == 0 && (uintptr_t)g.C % 16 == 0) ? 1 : 0;
    const int tiles_m = (g.M + GBM - 1) / GBM;
    int tiles_n = (g.N + GBN - 1) / GBN;
    a.seg_len = g.batch > 1 ? g.seg_len : 0;
    a.seg_stride = g.seg_stride;
    a.batch_c = g.batch_c;
    double flops = 2.0 * g.M * g.N * g.K, bytes = gemm_algorithmic_bytes<T>(g);
    if (g.B2.ptr) {
        // the second product of a segmented launch; the tile order below must keep an entry's tiles within one band
        if (a.seg_len <= 0 || !g.A.trans || !g.B.trans || !g.B2.trans || g.B2.packed || !g.C2 || g.N2 <= 0 || splits > 1 || g.bias ||
            tiles_m > 8) {
            set_error("gemm_blocked: a second product needs the batched rows-are-K form without split K, at most %d rows", 8 * GBM);
            return LSTM_ERR_UNSUPPORTED;
        }
        a.B2 = g.B2.ptr; a.C2 = g.C2; a.N2 = g.N2; a.ldb2 = g.B2.ncb; a.ldc2 = g.ldc2;
        a.tiles_n1 = tiles_n;
        tiles_n += (g.N2 + GBN - 1) / GBN;
        if (!(g.ldc2 % 8 == 0 && (uintptr_t)g.C2 % 16 == 0)) a.vec_out = 0;
        flops += 2.0 * g.M * g.N2 * g.K;
        bytes += (double)g.N2 * g.K * sizeof(T) + (double)g.M * g.N2 * (g.out_lp ? sizeof(T) : 4.0);
    }
    const dim3 grid(tiles_m * tiles_n, g.batch > 1 ? g.batch : 1, splits);
    KernelTimer timer(g.kclass, stream, flops, bytes);
    if (!g.A.trans && !g.B.trans)
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, false, false, true, true>), grid, dim3(GTHREADS), 0, stream, a, tiles_m, tiles_n);
    else if (!g.A.trans && g.B.trans)
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, false, true, true, true>), grid, dim3(GTHREADS), 0, stream, a, tiles_m, tiles_n);
    else if (g.A.trans && g.B.trans && a.seg_len > 0)
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, true, true, true, true, true>), grid, dim3(GTHREADS), 0, stream, a, tiles_m, tiles_n);
    else if (g.A.trans && g.B.trans)
        hipLaunchKernelGGL((gemm_mfma_big_kernel<T, true, true, true, true>), grid, dim3(GTHREADS), 0, stream, a, tiles_m, tiles_n);
    else {
        set_error("gemm_blocked: operand roles (A transposed, B not) have no kernel");
        return LSTM_ERR_UNSUPPORTED;
    }
    LSTM_LAUNCH_CHECK();
    GemmArgs r{};
    r.M = g.M; r.N = g.N; r.C = g.C; r.ldc = g.ldc; r.out_lp = g.out_lp; r.accumulate = g.accumulate; r.splitk_ws = g.splitk_ws;
    return finish_splitk<T>(r, splits, stream);
}
}  // namespace

size_t blocked_elems(int rows, int cols) { return (size_t)((rows + 63) / 64) * ((cols + 63) / 64) * 4096; }

int pack_blocked(int dtype, const void *src, int64_t ld, int rows, int cols, void *dst, hipStream_t stream) {
    if (rows <= 0 || cols <= 0) return LSTM_OK;
    const int nrb = (rows + 63) / 64, ncb = (cols + 63) / 64;
    if (nrb > 65535) {
        set_error("pack_blocked: too many rows %d", rows);
        return LSTM_ERR_UNSUPPORTED;
    }
    KernelTimer timer(KC_AUX, stream, 0.0, 0.0);
    if (dtype == LSTM_DTYPE_FP32)
        hipLaunchKernelGGL(pack_blocked_kernel<uint32_t>, dim3(ncb, nrb), dim3(256), 0, stream, (const uint32_t *)src, ld, rows, cols, (uint32_t *)dst, ncb);
    else if (ld % 8 == 0 && cols % 8 == 0 && ((uintptr_t)src | (uintptr_t)dst) % 16 == 0)
        hipLaunchKernelGGL(pack_blocked_vec_kernel, dim3(ncb, nrb), dim3(256), 0, stream, (const uint16_t *)src, ld, rows, cols, (uint16_t *)dst, ncb);
    else
        hipLaunchKernelGGL(pack_blocked_kernel<uint16_t>, dim3(ncb, nrb), dim3(256), 0, stream, (const uint16_t *)src, ld, rows, cols, (uint16_t *)dst, ncb);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

bool gemm_blocked_supported(int dtype, int M, int N) { return dtype != LSTM_DTYPE_FP32 && M >= 192 && N >= 192; }

int gemm_blocked(int dtype, const BlockedGemmArgs &g, hipStream_t stream) {
    if (!g.A.ptr || !g.B.ptr || !g.C || g.M < 1 || g.N < 1 || g.K < 1 || dtype == LSTM_DTYPE_FP32 || g.A.packed || g.B.packed) {
        set_error("gemm_blocked: invalid argument");
        return LSTM_ERR_INVALID;
    }
    int64_t kb = (g.K + 63) / 64;
    if (g.batch > 1) {
        // a batch of products whose K rows interleave in memory: whole segments, rows-are-K roles, no split-K
        if (!g.A.trans || !g.B.trans || g.seg_len < 1 || g.seg_stride < g.seg_len * g.batch || g.K % (64 * g.seg_len) != 0 ||
            g.splits > 1 || g.batch > 65535) {
            set_error("gemm_blocked: unsupported batched form (batch=%d seg_len=%d seg_stride=%d K=%d)", g.batch, g.seg_len,
                      g.seg_stride, g.K);
            return LSTM_ERR_UNSUPPORTED;
        }
        kb = kb / g.seg_len * g.seg_stride;            // block rows the batch spans in memory
    }
    // operand extents in elements must fit the kernel's 32-bit offsets
    const int64_t ea = (g.A.trans ? kb : (int64_t)(g.M + 63) / 64) * g.A.ncb * 4096;
    const int64_t eb = (g.B.trans ? kb : (int64_t)(g.N + 63) / 64) * g.B.ncb * 4096;
    const int64_t eb2 = g.B2.ptr ? kb * g.B2.ncb * 4096 : 0;
    if (ea >= (int64_t)1 << 31 || eb >= (int64_t)1 << 31 || eb2 >= (int64_t)1 << 31) {
        set_error("gemm_blocked: operand too large for 32-bit offsets");
        return LSTM_ERR_UNSUPPORTED;
    }
    return dtype == LSTM_DTYPE_FP16 ? launch_blocked<_Float16>(g, stream) : launch_blocked<bf16_t>(g, stream);
}

bool gemm_tn_supported(int dtype, const GemmArgs &g) {
    return dtype != LSTM_DTYPE_FP32 && g.M % 8 == 0 && g.N % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
           (uintptr_t)g.A % 16 == 0 && (uintptr_t)g.B % 16 == 0 && g.M >= 192 && g.N >= 192 && g.K >= 1 &&
           fits_32bit(g.K, g.lda, g.K, g.ldb);
}

int gemm_tn(int dtype, const GemmArgs &g, hipStream_t stream) {
    if (!gemm_tn_supported(dtype, g)) {
        set_error("gemm_tn: unsupported shape or alignment (M=%d N=%d K=%d)", g.M, g.N, g.K);
        return LSTM_ERR_UNSUPPORTED;
    }
    if (!g.A || !g.B || !g.C) {
        set_error("gemm_tn: null operand");
        return LSTM_ERR_INVALID;
    }
    return dtype == LSTM_DTYPE_FP16 ? launch_tn<_Float16>(g, stream) : launch_tn<bf16_t>(g, stream);
}

// Diagnostic: register-resident MFMA loop (no memory traffic inside the loop), the rate the matrix
// pipes sustain on the given operand values.  256 workgroups x 8 wavefronts, 8 independent 32x32
// accumulators per wavefront; every lane takes its two fragments from `operands`.
namespace {
template <typename T>
__global__ __launch_bounds__(512) void mfma_rate_kernel(const u32x4 *operands, int iters, float *sink) {
    const u32x4 fa = operands[(blockIdx.x * 512 + threadIdx.x) * 2];
    const u32x4 fb = operands[(blockIdx.x * 512 + threadIdx.x) * 2 + 1];
    v16f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = Lp<T>::mfma(fa, fb, acc[j]);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    if (s == 12345.678f) sink[0] = s;              // keeps the loop alive; practically never taken
}
}  // namespace

int mfma_rate(int dtype, const void *operands, int iters, float *sink, double *flops, hipStream_t stream) {
    if (dtype == LSTM_DTYPE_FP32 || !operands || !sink || iters < 1 || iters > (1 << 22)) {
        set_error("mfma_rate: 16-bit type, operands, sink and 1 <= iters <= 2^22 required");
        return LSTM_ERR_INVALID;
    }
    if (dtype == LSTM_DTYPE_FP16)
        hipLaunchKernelGGL(mfma_rate_kernel<_Float16>, dim3(256), dim3(512), 0, stream, (const u32x4 *)operands, iters, sink);
    else
        hipLaunchKernelGGL(mfma_rate_kernel<bf16_t>, dim3(256), dim3(512), 0, stream, (const u32x4 *)operands, iters, sink);
    LSTM_LAUNCH_CHECK();
    if (flops) *flops = 256.0 * 8.0 * 8.0 * (double)iters * 2.0 * 32.0 * 32.0 * 16.0;
    return LSTM_OK;
}

}  // namespace lstm
