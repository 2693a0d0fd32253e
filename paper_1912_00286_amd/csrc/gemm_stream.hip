// C[M,N] (+ bias) = A B^T for the whole-sequence products of wide layers whose operands exist in packed
// (MFMA-fragment) order anyway: A = the packed per-time-step copies the recurrent kernels read (h_t resp.
// dA_t), B = a weight matrix packed like the recurrent kernels' B operand (packed.h).
//
// What this kernel is built around (all measured on this part):
//   * On real (non-constant) operands the matrix rate is set by the power cap, and the 16x16x32 MFMA moves half as
//     many accumulator registers per flop as the 32x32x16 one (register-resident loops: 2.03 against 1.70
//     PFLOP/s on N(0,1) operands): 16x16x32 throughout.
//   * The matrix pipe holds one MFMA besides the one it executes.  Whatever else a wavefront issues has to go
//     between two MFMAs one instruction at a time; a batch of LDS reads or loads leaves the pipe idle.  The K loop
//     is therefore written out in issue order: two MFMAs, one LDS read, ... with a scheduling barrier after every
//     such group, and the MFMAs as inline assembly with their accumulators pinned to the accumulator registers
//     (left to itself the compiler keeps a few of the 64 accumulator tuples elsewhere and moves them in and out
//     between MFMAs).
//   * Nothing is staged through registers.  A workgroup of four wavefronts (one per SIMD) owns 256 x 256 of C,
//     wavefront w rows 64 w .. 64 w + 63 over all 256 columns.  The A fragments of a wavefront's rows are needed by
//     nobody else: they go from memory straight into the registers the MFMA reads (a ring of four K chunks).  The B
//     chunk (256 rows x 64 k = 32 KB), which all four need, is fetched once per workgroup with direct-to-LDS loads
//     into a ring of four stages, already in fragment order: a fragment read is contiguous per 16-lane group, free
//     of bank conflicts without padding.  One workgroup barrier per K chunk; the first fragments of the next chunk
//     are read ahead of it.
// The K loop is unrolled over groups of four chunks with a branch-free body (ring slots and outstanding-load
// counts are compile-time constants); K must be a multiple of 256.
#include "kernels.h"
#include "packed.h"

namespace lstm {
namespace {

typedef __attribute__((address_space(3))) void *lds_ptr;

constexpr int SG_THREADS = 256;
constexpr int SG_NS = 4;                          // LDS stages = register sets: chunk c lives in slot c % 4
constexpr int SG_STAGE = 2 * B_CHUNK * 2;         // bytes of one stage: two packed B tiles' chunk (32 KB)
constexpr int SG_OLD = 256 + 8;                   // row pitch (elements) of the staged result tile
constexpr int SG_LDS = SG_NS * SG_STAGE > 256 * SG_OLD * 2 ? SG_NS * SG_STAGE : 256 * SG_OLD * 2;
constexpr int SG_GRP = 4;                         // chunks per unrolled group (a multiple of SG_NS)

struct StreamArgs {
    const uint16_t *A;        // packed rows: time step s at A + s * a_step_stride, there [row tile][nkc][A_CHUNK]
    int64_t a_step_stride;    // elements
    int tiles_per_step;       // 64-row tiles per time step
    const uint16_t *Bpk;      // [B tile of 128 rows][nkc][B_CHUNK]
    int n_btiles;
    void *C;                  // 16-bit, row-major [M, ldc]
    int64_t ldc;
    const void *bias;         // [N] or null
    int M, N, nkc;
    int gate_h;               // 0: B row n is column n.  H > 0: B tile j, row 32 g + r is column g H + 32 j + r
    int tiles_m, tiles_n;
};

// direct-to-LDS load of 16 bytes per lane; piece p of eight lies (p - 4) KB from both bases
__device__ __forceinline__ void sg_dma_piece(const void *src, lds_ptr dst, int p) {
    switch (p) {
        case 0: __builtin_amdgcn_global_load_lds(src, dst, 16, -4096, 0); break;
        case 1: __builtin_amdgcn_global_load_lds(src, dst, 16, -3072, 0); break;
        case 2: __builtin_amdgcn_global_load_lds(src, dst, 16, -2048, 0); break;
        case 3: __builtin_amdgcn_global_load_lds(src, dst, 16, -1024, 0); break;
        case 4: __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 0); break;
        case 5: __builtin_amdgcn_global_load_lds(src, dst, 16, 1024, 0); break;
        case 6: __builtin_amdgcn_global_load_lds(src, dst, 16, 2048, 0); break;
        default: __builtin_amdgcn_global_load_lds(src, dst, 16, 3072, 0); break;
    }
}

// c += a b on the 16x16x32 matrix instruction with the accumulator pinned to the accumulator registers
template <typename T> __device__ __forceinline__ void mfma_acc(v4f &c, const u32x4 &x, const u32x4 &y);
template <> __device__ __forceinline__ void mfma_acc<_Float16>(v4f &c, const u32x4 &x, const u32x4 &y) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
}
template <> __device__ __forceinline__ void mfma_acc<bf16_t>(v4f &c, const u32x4 &x, const u32x4 &y) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
}

template <int N> __device__ __forceinline__ void sg_wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <typename T>
__global__ __launch_bounds__(SG_THREADS) void gemm_stream_kernel(StreamArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char ring[SG_LDS];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // tile order: workgroups of one XCD (id % 8) take neighbouring tiles, walked in bands of 8 tile rows so that
    // a band's A and B panels stay in that XCD's L2
    const int total = a.tiles_m * a.tiles_n;
    int lin = blockIdx.x;
    if (total % 8 == 0) lin = (lin % 8) * (total / 8) + lin / 8;
    const int band = 8 * a.tiles_n;
    const int b0 = (lin / band) * 8;
    const int bh = min(8, a.tiles_m - b0);
    const int tm = b0 + (lin % band) % bh, tn = (lin % band) / bh;

    // this wavefront's 64 rows of A = one packed row tile (tiles past the end are read from tile 0 and never stored)
    const int row_tiles = a.M / 64;
    const int rt = tm * 4 + wave, rtc = rt < row_tiles ? rt : 0;
    // (wavefront-uniform base addresses; the lane's 16 bytes are added as a 32-bit offset at the access, which
    // lets a load take its address from scalar registers + one vector register + an immediate)
    const char *Aw = reinterpret_cast<const char *>(a.A + (int64_t)(rtc / a.tiles_per_step) * a.a_step_stride +
                                                    (int64_t)(rtc % a.tiles_per_step) * a.nkc * A_CHUNK);
    const unsigned lane16 = lane * 16;
    // its eight 1 KB pieces of every B stage: pieces 8 w .. 8 w + 7 of 32 (the first 16 belong to B tile 2 tn)
    const int bt = 2 * tn + (wave >> 1), btc = bt < a.n_btiles ? bt : 0;
    const char *Bw = reinterpret_cast<const char *>(a.Bpk + (int64_t)btc * a.nkc * B_CHUNK + (wave & 1) * 8 * 64 * 8);
    unsigned char *my_pieces = ring + wave * 8192;

    // 16x16x32 MFMA: block (i, f) of this wavefront's 64 x 256 = rows 16 i.., columns 16 f..
    v4f acc[4][16];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int f = 0; f < 16; ++f)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][f][r] = 0.0f;
    // Operand fragments of the 16x16x32 form out of the 32-row fragment order: lane = 16 (k / 8) + row, k-group kg =
    // lane / 16 of the 32-deep step lies in 16-deep step kg / 2, half kg % 2 of the stored order.
    const int frow = lane & 15, kg = lane >> 4;
    const unsigned laneA = (kg >> 1) * 2048 + ((kg & 1) * 32 + frow) * 16;   // + (q * 4 + (i >> 1)) * 1024 + (i & 1) * 256
    const unsigned laneB = (kg >> 1) * 4096 + ((kg & 1) * 32 + frow) * 16;   // + tile * 16384 + q * 8192 + blk * 1024 + sub * 256
    u32x4 areg[SG_NS][8];                                // chunk c in slot c % 4: fragment (32-deep step q, 16-row block i) at [4 q + i]
    u32x4 bf[2][8];                                      // B fragments of column blocks 0..7 (B tile 0) in bf[0], 8..15 in bf[1]

    auto read_b = [&](u32x4 (&b)[8], int st, int q, int tile) {
        const unsigned char *p = ring + st * SG_STAGE + tile * 16384 + q * 8192 + laneB;
#pragma unroll
        for (int f = 0; f < 8; ++f) b[f] = *reinterpret_cast<const u32x4 *>(p + (f >> 1) * 1024 + (f & 1) * 256);
    };
    // half of a 32-deep step: 32 MFMAs on eight column blocks.  The matrix pipe holds one MFMA besides the one it
    // executes, so everything else goes between MFMAs one instruction at a time: first the 8 B fragments of the next
    // half (other register set), then four of the chunk's memory requests (B pieces of chunk cb, or A fragments into
    // registers `arl` that the 32-deep step before has left)
    auto half32 = [&](const u32x4 (&ar)[8], int q, int tile, int stn, int qn, const char *srcB, unsigned char *dstB, int pb,
                      u32x4 (&arl)[8], int ql, const char *srcA) {
        const unsigned char *pn = ring + stn * SG_STAGE + (tile ^ 1) * 16384 + qn * 8192 + laneB;
        // MFMA n of the half: column block tile * 8 + n / 4, row block n % 4
        auto mm = [&](int n) { mfma_acc<T>(acc[n & 3][tile * 8 + (n >> 2)], ar[q * 4 + (n & 3)], bf[tile][n >> 2]); };
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            mm(2 * j);
            mm(2 * j + 1);
            bf[tile ^ 1][j] = *reinterpret_cast<const u32x4 *>(pn + (j >> 1) * 1024 + (j & 1) * 256);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
#pragma unroll
            for (int n = 0; n < 4; ++n) mm(16 + 4 * m + n);
            if (pb >= 0) sg_dma_piece(srcB + lane16, (lds_ptr)dstB, pb + m);
            else arl[ql * 4 + m] = *reinterpret_cast<const u32x4 *>(srcA + laneA + (ql * 4 + (m >> 1)) * 1024 + (m & 1) * 256);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto issueA = [&](u32x4 (&ar)[8], int c, int q) {
        const char *src = Aw + (int64_t)c * (A_CHUNK * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) ar[q * 4 + i] = *reinterpret_cast<const u32x4 *>(src + laneA + (q * 4 + (i >> 1)) * 1024 + (i & 1) * 256);
    };
    auto issueB = [&](int c, int st) {
        const char *src = Bw + (int64_t)c * (B_CHUNK * 2);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            __builtin_amdgcn_global_load_lds(reinterpret_cast<const u32x4 *>(src + lane16 + i * 1024), (lds_ptr)(my_pieces + st * SG_STAGE + i * 1024), 16, 0, 0);
    };

    // Per wavefront and step: 8 B pieces (direct to LDS) and 8 A fragments (registers); a wavefront's loads complete
    // in issue order.  Step c multiplies chunk c and requests B(c+3) into the stage chunk c - 1 occupied, the second
    // half of A(c+3) into the registers the second half of chunk c - 1 occupied, and the first half of A(c+4) into
    // the registers its own first half leaves.  It ends with [wait until at most its own 16 requests are outstanding:
    // everything requested before this step has landed] [barrier: chunk c + 2 is complete in LDS, everybody is done
    // with chunk c].  Requests past the last chunk are clamped to the last one (never read).
    const int last = a.nkc - 1;
    issueA(areg[0], 0, 0); issueA(areg[0], 0, 1);
    issueB(0, 0);
    issueA(areg[1], 1, 0); issueA(areg[1], 1, 1);
    issueB(1, 1);
    issueA(areg[2], 2, 0);
    __builtin_amdgcn_sched_barrier(0);
    issueB(2, 2);
    issueA(areg[2], 2, 1);
    issueA(areg[3], 3, 0);
    __builtin_amdgcn_sched_barrier(0);
    sg_wait_vm<16>();
    __builtin_amdgcn_s_barrier();
    read_b(bf[0], 0, 0, 0);
    for (int g = 0; g <= last; g += SG_GRP) {
#pragma unroll
        for (int i = 0; i < SG_GRP; ++i) {
            const int c = g + i;
            const int cb = c + 3 < last ? c + 3 : last, c4 = c + 4 < last ? c + 4 : last;
            const char *srcB = Bw + (int64_t)cb * (B_CHUNK * 2) + 4096;
            unsigned char *dstB = my_pieces + ((i + 3) % SG_NS) * SG_STAGE + 4096;
            // 32-deep step 0: B pieces 0..3, then the second-half A fragments of chunk c + 3 (slot of chunk c - 1)
            half32(areg[i % SG_NS], 0, 0, i % SG_NS, 0, srcB, dstB, 0, areg[(i + 3) % SG_NS], 1, nullptr);
            half32(areg[i % SG_NS], 0, 1, i % SG_NS, 1, srcB, dstB, -1, areg[(i + 3) % SG_NS], 1, Aw + (int64_t)cb * (A_CHUNK * 2));
            // 32-deep step 1: B pieces 4..7, then the first-half A fragments of chunk c + 4 (this chunk's slot)
            half32(areg[i % SG_NS], 1, 0, i % SG_NS, 1, srcB, dstB, 4, areg[i % SG_NS], 0, nullptr);
            half32(areg[i % SG_NS], 1, 1, (i + 1) % SG_NS, 0, srcB, dstB, -1, areg[i % SG_NS], 0, Aw + (int64_t)c4 * (A_CHUNK * 2));
            sg_wait_vm<16>();
            __builtin_amdgcn_s_barrier();
        }
    }
    sg_wait_vm<0>();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last MFMAs leave the pipe before their accumulators are read
    __syncthreads();                                     // every stage is free: the ring becomes the staged result tile

    // 16-bit result: stage the tile (bias added) and write whole 128-byte row segments
    T *stage = reinterpret_cast<T *>(ring);
    const T *bias = reinterpret_cast<const T *>(a.bias);
    const int col_l = lane & 15, rgrp = (lane >> 4) * 4;
#pragma unroll
    for (int f = 0; f < 16; ++f) {
        // B row of column block f: tile f / 8, 32-row block (f % 8) / 2, half f % 2.  Staged column order: gate-major
        // when the B rows interleave gates, so that a row's segments are contiguous in C
        const int tile = f >> 3, blk = (f & 7) >> 1, sub = f & 1;
        const int sc = a.gate_h ? (blk * 2 + tile) * 32 + sub * 16 + col_l : f * 16 + col_l;
        const int unit = (2 * tn + tile) * 32 + sub * 16 + col_l;
        const int col = a.gate_h ? blk * a.gate_h + unit : tn * 256 + f * 16 + col_l;
        const bool col_ok = a.gate_h ? unit < a.gate_h : col < a.N;
        const float bv = (bias && col_ok) ? Lp<T>::to_f(bias[col]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rl = wave * 64 + i * 16 + rgrp + r;
                stage[rl * SG_OLD + sc] = Lp<T>::from_f(acc[i][f][r] + bv);
            }
    }
    __syncthreads();
    T *C = reinterpret_cast<T *>(a.C);
#pragma unroll 4
    for (int v = tid; v < 256 * 32; v += SG_THREADS) {
        const int rl = v >> 5, cv = v & 31;
        const int row = tm * 256 + rl;
        int col;
        bool ok;
        if (a.gate_h) {
            const int unit = tn * 64 + (cv & 7) * 8;
            col = (cv >> 3) * a.gate_h + unit;
            ok = unit < a.gate_h;
        } else {
            col = tn * 256 + cv * 8;
            ok = col < a.N;
        }
        if (row >= a.M || !ok) continue;
        *reinterpret_cast<u32x4 *>(&C[(int64_t)row * a.ldc + col]) = *reinterpret_cast<const u32x4 *>(&stage[rl * SG_OLD + cv * 8]);
    }
}

}  // namespace

bool gemm_stream_supported(int dtype, const StreamGemmArgs &g) {
    if (dtype == LSTM_DTYPE_FP32) return false;
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
    if (g.M % 64 != 0 || g.K % (64 * SG_GRP) != 0 || g.N % 8 != 0 || g.ldc % 8 != 0) return false;
    if (g.rows_per_step <= 0 || g.rows_per_step % 64 != 0 || g.M % g.rows_per_step != 0) return false;
    if (g.gate_h != 0 && (g.gate_h % 32 != 0 || g.N != 4 * g.gate_h)) return false;
    return true;
}

int gemm_stream(int dtype, const StreamGemmArgs &g, hipStream_t stream) {
    if (!gemm_stream_supported(dtype, g)) {
        set_error("gemm_stream: unsupported shape M=%d N=%d K=%d rows/step=%d (16-bit types, M and rows per step multiples of 64, "
                  "K a multiple of %d)", g.M, g.N, g.K, g.rows_per_step, 64 * SG_GRP);
        return LSTM_ERR_INVALID;
    }
    if (!g.A || !g.B || !g.C || (uintptr_t)g.A % 16 || (uintptr_t)g.B % 16 || (uintptr_t)g.C % 16 || g.a_step_stride % 8) {
        set_error("gemm_stream: null or misaligned operand");
        return LSTM_ERR_INVALID;
    }
    StreamArgs a{};
    a.A = (const uint16_t *)g.A; a.a_step_stride = g.a_step_stride; a.tiles_per_step = g.rows_per_step / 64;
    a.Bpk = (const uint16_t *)g.B;
    a.n_btiles = g.gate_h ? g.gate_h / 32 : (g.N + 127) / 128;
    a.C = g.C; a.ldc = g.ldc; a.bias = g.bias;
    a.M = g.M; a.N = g.N; a.nkc = g.K / 64; a.gate_h = g.gate_h;
    a.tiles_m = (g.M + 255) / 256;
    a.tiles_n = g.gate_h ? (g.gate_h + 63) / 64 : (g.N + 255) / 256;
    const double flops = 2.0 * g.M * g.N * g.K;
    const double bytes = 2.0 * ((double)g.M * g.K + (double)g.N * g.K + (double)g.M * g.N);
    KernelTimer timer(g.kclass, stream, flops, bytes);
    const dim3 grid(a.tiles_m * a.tiles_n);
    if (dtype == LSTM_DTYPE_FP16) hipLaunchKernelGGL(gemm_stream_kernel<_Float16>, grid, dim3(SG_THREADS), 0, stream, a);
    else hipLaunchKernelGGL(gemm_stream_kernel<bf16_t>, grid, dim3(SG_THREADS), 0, stream, a);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace lstm
