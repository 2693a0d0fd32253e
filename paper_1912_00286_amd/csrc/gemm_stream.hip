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
#include <type_traits>

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
    // A lane's 16 bytes of a 1 KB piece of a B stage.  The piece is [k half][row 0 .. 31 of a 32-row block]; the LDS
    // image keeps that shape but holds row 8 (i / 4) + 4 s + i % 4 of the block in slot 16 s + i (s = 0, 1; i = 0 .. 15),
    // by letting the lane of that slot fetch that row: the 16-row fragment s of the block then holds, at MFMA index
    // 4 g + r, column 8 g + 4 s + r of the block's 32, so that the two fragments' accumulators of a lane are 8
    // consecutive columns of C (see the result stores below).
    const int slot = lane & 31;
    const unsigned lane16 = (unsigned)(((lane & 32) + 8 * ((slot & 15) >> 2) + 4 * (slot >> 4) + (slot & 3)) * 16);
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
        // MFMA n of the half: column block tile * 8 + n / 4, row block n % 4.  The B fragment is the first operand: a
        // lane's four accumulator values are then four columns of one row of C
        auto mm = [&](int n) { mfma_acc<T>(acc[n & 3][tile * 8 + (n >> 2)], bf[tile][n >> 2], ar[q * 4 + (n & 3)]); };
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
    // 16-bit result (bias added) straight from the accumulators.  Lane (m = lane % 16, g = lane / 16) holds, of the
    // 32-column group p = (B tile p / 4, 32-row block p % 4) and row block i, columns 8 g .. 8 g + 3 in the group's
    // first fragment and 8 g + 4 .. 8 g + 7 in its second, all of row 16 i + m: 16 bytes, and the four lanes of a row
    // 64 consecutive bytes.  Stores want whole 128-byte lines (half lines were measured at a third of the rate), so
    // two groups that are neighbours in C are written together: lanes m < 8 and m >= 8 swap one group's values
    // (lane m with lane m ^ 8, a rotation by 8 inside the row of 16 lanes), after which one store instruction covers
    // rows 0 .. 7 of the block and the next rows 8 .. 15, 128 bytes each.
    T *C = reinterpret_cast<T *>(a.C);
    const T *bias = reinterpret_cast<const T *>(a.bias);
    const int ml = lane & 15, g8 = (lane >> 4) * 8;
    const bool lo = ml < 8;
    const int row0 = tm * 256 + wave * 64 + (ml & 7);
    // groups pa and pb = pa's right-hand neighbour; col: first column of the lane's 8 in group pa
    auto store_pair = [&](auto pa_c, auto pb_c, int col, int colb, bool oka, bool okb) {
        constexpr int pa = decltype(pa_c)::value, pb = decltype(pb_c)::value;
        __attribute__((aligned(16))) T bla[8], blb[8];
        if (bias && oka) *reinterpret_cast<u32x4 *>(bla) = *reinterpret_cast<const u32x4 *>(bias + col);
        if (bias && okb) *reinterpret_cast<u32x4 *>(blb) = *reinterpret_cast<const u32x4 *>(bias + colb);
        float bva[8], bvb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            bva[e] = (bias && oka) ? Lp<T>::to_f(bla[e]) : 0.0f;
            bvb[e] = (bias && okb) ? Lp<T>::to_f(blb[e]) : 0.0f;
        }
        const bool ok = lo ? oka : okb;                  // of the group this lane stores
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __attribute__((aligned(16))) T oa[8], ob[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                oa[r] = Lp<T>::from_f(acc[i][2 * pa][r] + bva[r]);
                oa[4 + r] = Lp<T>::from_f(acc[i][2 * pa + 1][r] + bva[4 + r]);
                ob[r] = Lp<T>::from_f(acc[i][2 * pb][r] + bvb[r]);
                ob[4 + r] = Lp<T>::from_f(acc[i][2 * pb + 1][r] + bvb[4 + r]);
            }
            const u32x4 va = *reinterpret_cast<const u32x4 *>(oa), vb = *reinterpret_cast<const u32x4 *>(ob);
            u32x4 got;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                got[d] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(lo ? vb[d] : va[d]), 0x128, 0xf, 0xf, false);   // row_ror:8
            // rows 0 .. 7: own group pa (m < 8) | the partner's group pb; rows 8 .. 15: the partner's pa | own pb
            const int c = lo ? col : colb;
            const int r0 = row0 + i * 16;
            if (ok && r0 < a.M) *reinterpret_cast<u32x4 *>(&C[(int64_t)r0 * a.ldc + c]) = lo ? va : got;
            if (ok && r0 + 8 < a.M) *reinterpret_cast<u32x4 *>(&C[(int64_t)(r0 + 8) * a.ldc + c]) = lo ? got : vb;
        }
    };
    if (a.gate_h) {
        // B tile j, row 32 g + r is column g H + 32 j + r: the neighbour of (tile 0, block b) is (tile 1, block b)
        const int unit = 2 * tn * 32 + g8;
        const bool oka = unit < a.gate_h, okb = unit + 32 < a.gate_h;
        store_pair(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{}, unit, unit + 32, oka, okb);
        store_pair(std::integral_constant<int, 1>{}, std::integral_constant<int, 5>{}, a.gate_h + unit, a.gate_h + unit + 32, oka, okb);
        store_pair(std::integral_constant<int, 2>{}, std::integral_constant<int, 6>{}, 2 * a.gate_h + unit, 2 * a.gate_h + unit + 32, oka, okb);
        store_pair(std::integral_constant<int, 3>{}, std::integral_constant<int, 7>{}, 3 * a.gate_h + unit, 3 * a.gate_h + unit + 32, oka, okb);
    } else {
        const int col = tn * 256 + g8;
        store_pair(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}, col, col + 32, col < a.N, col + 32 < a.N);
        store_pair(std::integral_constant<int, 2>{}, std::integral_constant<int, 3>{}, col + 64, col + 96, col + 64 < a.N, col + 96 < a.N);
        store_pair(std::integral_constant<int, 4>{}, std::integral_constant<int, 5>{}, col + 128, col + 160, col + 128 < a.N, col + 160 < a.N);
        store_pair(std::integral_constant<int, 6>{}, std::integral_constant<int, 7>{}, col + 192, col + 224, col + 192 < a.N, col + 224 < a.N);
    }
}

// ---------------------------------------------------------------- C = A^T B, both operands with the contraction index as rows
// The weight gradients dW = dA^T X, dU = dA^T H: both operands are 64x64-blocked activations whose rows are the
// contraction index (all T*B rows), so the fragments have to be transposed on the way into the MFMA, which the LDS
// transpose read does: both operands go through LDS.  Same loop as above (16x16x32 MFMAs pinned to the accumulator
// registers, one other instruction between two MFMAs, four stages, fragments of the next step read ahead of the
// barrier), with these differences:
//   * a stage is 32 contraction rows x (256 m + 256 n): 32 KB, so that four of them fit; the rows of a blocked
//     operand are whole 128-byte lines, so half a 64x64 block is still fetched in whole lines;
//   * both operands arrive by direct-to-LDS loads, 1 KB (8 rows of one block) per wavefront instruction;
//   * four wavefronts of 128 x 128 each (2 x 2): 8 A and 8 B fragments per 32-deep step, two 8-byte transpose
//     reads each;
//   * the LDS image keeps the rows at their 128-byte pitch and swaps 32-byte groups inside a row, group' = group ^
//     f(row), f = bit 1 of the row | bit 3 of the row << 1: the sixteen rows one transpose-read instruction touches
//     (rows 8 g .. 8 g + 3 of its four 16-lane groups g) then spread evenly over the banks.  The swap is applied by
//     choosing which 16 bytes each lane of a direct-to-LDS load fetches.
// Operand formats: 64x64 blocks [K / 64][ncb][64][64] (row-major inside a block), or (PK) the packed copies the
// recurrent kernels write, kept for all time steps one after the other: [K / 64][ncb][64 x 64 in fragment order,
// packed.h].  Either way 64 contraction rows x 64 columns are 8 KB and a row's 8 columns are 16 contiguous bytes;
// only the place of those 16 bytes inside the 8 KB differs.  The packed form keeps that order in LDS too (see the
// loads in the kernel), with the transpose reads addressed accordingly.
struct StreamTnArgs {
    const uint16_t *A;        // rows = contraction index, columns = m (first m block at column block 0)
    const uint16_t *B;        // columns = n
    int ncb_a, ncb_b;
    void *C;                  // 16-bit, row-major [M, ldc]
    int64_t ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    float *ws;                // split K: fp32 partial results [split][M][N] (the caller adds them up), else null
    int split_steps;          // 32-row steps per split (K / 32 without split K)
};

typedef short sg_v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) sg_v4s *sg_lds_v4s;

// Direct-to-LDS load of 16 bytes per lane: global address = base (scalar) + offset (per lane) + j KB, LDS address =
// lds + 16 lane + j KB.  Written as assembly because the compiler, once it has seen a direct-to-LDS load, waits for
// ALL outstanding loads before every LDS transpose read that follows (it cannot tell the two apart), which would
// serialise the whole pipeline; the waits these loads need are the explicit ones of the loop.  M0 carries the LDS
// address (nothing else in the kernel uses it).
template <bool PK>
__device__ __forceinline__ void sg_dma_piece4(const void *base, unsigned offset, unsigned lds, int j) {
    if constexpr (PK) {
        // packed source: a piece is the kilobyte of one 16-column group (32 rows x 2 halves of 8 columns); the next
        // group lies 2 KB further on in memory (scalar base) and 1 KB further on in LDS (M0)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(offset), "s"(reinterpret_cast<const char *>(base) + 2048 * j), "s"(lds + 1024u * j) : "memory");
        return;
    }
    switch (j) {
        case 0: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(offset), "s"(base), "s"(lds) : "memory"); break;
        case 1: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024" :: "v"(offset), "s"(base), "s"(lds) : "memory"); break;
        case 2: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048" :: "v"(offset), "s"(base), "s"(lds) : "memory"); break;
        default: asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072" :: "v"(offset), "s"(base), "s"(lds) : "memory"); break;
    }
}

template <typename T, bool PK>
__global__ __launch_bounds__(SG_THREADS) void gemm_stream_tn_kernel(StreamTnArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char ring[SG_LDS];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int total = a.tiles_m * a.tiles_n;
    const int split = (int)blockIdx.x / total;            // split K: the workgroups of one split follow each other
    int lin = (int)blockIdx.x - split * total;
    if (total % 8 == 0) lin = (lin % 8) * (total / 8) + lin / 8;
    const int band = 8 * a.tiles_n;
    const int b0 = (lin / band) * 8;
    const int bh = min(8, a.tiles_m - b0);
    const int tm = b0 + (lin % band) % bh, tn = (lin % band) / bh;

    // Loads.  Piece p of a stage's 32: operand p / 16 (A, B), block (p / 4) % 4 of the tile's four, rows 8 (p % 4) ..
    // of the stage's 32.  Wavefront w takes pieces 8 w .. 8 w + 7: two blocks of one operand, four pieces each.
    // Lane i of a piece holds row i / 8 and the 16 bytes at position i % 8 of that row, and fetches the 16 bytes that
    // belong there under the swap: chunk (i % 8) ^ 2 f, f from the row 8 (p % 4) + i / 8 (two cases: p % 4 even, odd).
    const bool opB = wave >= 2;
    const uint16_t *Op = opB ? a.B : a.A;
    const int ncb = opB ? a.ncb_b : a.ncb_a, nblk = ((opB ? a.N : a.M) + 63) / 64;
    const int blk0 = (opB ? tn : tm) * 4 + (wave & 1) * 2;
    const int blkc0 = blk0 < nblk ? blk0 : 0, blkc1 = blk0 + 1 < nblk ? blk0 + 1 : 0;      // blocks past the edge: read block 0, never stored
    // Packed operands (PK) keep their own order in LDS instead: a piece is one 16-column group of a block, the
    // contiguous kilobyte [8-column half][row 0 .. 31][16 bytes], so that neighbouring lanes fetch neighbouring
    // memory (fetching the row-major image out of it would send the eight lanes of a row to eight different lines).
    // Only the rows of the second half are stored with bit 2 flipped (again by the choice of what a lane fetches):
    // the two halves one transpose read touches then fall on different banks.
    const int lrow = lane >> 3, lpos = lane & 7;
    // byte offset of (row lrow, 16-byte chunk ch) inside the 8 rows a piece covers
    auto chunk_off = [&](int ch) -> unsigned { return (unsigned)(lrow * 128 + ch * 16); };
    const unsigned lsrc_pk = (unsigned)(((lane & 32) + ((lane & 31) ^ ((lane >> 5) << 2))) * 16);
    const unsigned lsrc0 = PK ? lsrc_pk : chunk_off(lpos ^ ((((lrow >> 1) & 1) | 0) << 1));   // pieces with p % 4 even
    const unsigned lsrc1 = PK ? lsrc_pk : chunk_off(lpos ^ ((((lrow >> 1) & 1) | 2) << 1));   // pieces with p % 4 odd
    const int64_t row_bytes = (int64_t)ncb * 8192;                                             // one block row of the operand
    const int64_t split_off = (int64_t)split * (a.split_steps >> 1) * row_bytes;               // (a split is whole block rows)
    const char *src0 = reinterpret_cast<const char *>(Op + (int64_t)blkc0 * 4096) + split_off;  // + block row * ncb * 8 KB + half * 4 KB
    const char *src1 = reinterpret_cast<const char *>(Op + (int64_t)blkc1 * 4096) + split_off;
    unsigned char *my_pieces = ring + wave * 8192;
    // pieces q = 0 .. 7 of step c into stage st
    auto dma = [&](int c, int st, int q) {
        const char *s = (q < 4 ? src0 : src1) + (int64_t)(c >> 1) * row_bytes + (c & 1) * (PK ? 1024 : 4096);
        const unsigned lds = (unsigned)(uintptr_t)(lds_ptr)(my_pieces + st * SG_STAGE + (q >> 2) * 4096);
        sg_dma_piece4<PK>(s, (q & 1) ? lsrc1 : lsrc0, lds, q & 3);
    };

    // Fragments.  Lane (i = lane % 16, g = lane / 16) of a transpose read supplies the address of 4 columns of row
    // 8 g + i / 4 (+ 4 for the second read) and receives the four rows' values of column i: contraction values 8 g ..
    // 8 g + 7 of column i, the 16x16x32 operand layout.  f of those rows is the same for both reads.
    const int ti = lane & 15, tg = lane >> 4;
    const int tf = ((ti >> 3) & 1) | ((tg & 1) << 1);
    unsigned tr_off[4];                                   // 16-column group cp of a block: byte offset of this lane's first read
#pragma unroll
    for (int cp = 0; cp < 4; ++cp) tr_off[cp] = (8 * tg + (ti >> 2)) * 128 + ((cp ^ tf) << 5) + (ti & 3) * 8;
    // PK: group cp is the kilobyte cp; inside it [half = bit 1 of ti][row, bit 2 flipped in the second half][16 bytes],
    // and the second read (4 rows further on) is the same address with that row bit the other way round
    const int th = (ti >> 1) & 1;
    const unsigned tr_pk = (unsigned)(th * 512 + ((8 * tg + (ti >> 2)) ^ (th << 2)) * 16 + (ti & 1) * 8);
    const unsigned tr_pk2 = tr_pk ^ 64u;
    auto read_frag = [&](const unsigned char *blk, int cp) -> u32x4 {
        const sg_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((sg_lds_v4s)(blk + (PK ? tr_pk + cp * 1024 : tr_off[cp])));
        const sg_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((sg_lds_v4s)(blk + (PK ? tr_pk2 + cp * 1024 : tr_off[cp] + 512)));
        struct { sg_v4s l, h; } both = {lo, hi};
        return __builtin_bit_cast(u32x4, both);
    };

    v4f acc[8][8];                                        // block (ia, jb) of the wavefront's 128 x 128
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;
    u32x4 fa[2][8], fb[2][8];                             // fragments of step c in set c % 2
    // fragment x of a stage: x < 8: B fragment x, else A fragment x - 8 (B first: the MFMAs walk along jb)
    auto read_one = [&](int set, int st, int x) {
        if (x < 8) fb[set][x] = read_frag(ring + st * SG_STAGE + 16384 + (wn * 2 + (x >> 2)) * 4096, x & 3);
        else fa[set][x - 8] = read_frag(ring + st * SG_STAGE + (wm * 2 + ((x - 8) >> 2)) * 4096, x & 3);
    };

    // Step c multiplies the 32 contraction rows of stage c % 4 and requests step c + 3 into the stage step c - 1
    // occupied; it ends with [wait until at most its own 8 requests are outstanding] [barrier: step c + 2 is complete
    // in LDS, everybody is done with step c].  Requests past the last step are clamped to it (never read).
    const int last = a.split_steps - 1;
#pragma unroll
    for (int q = 0; q < 8; ++q) dma(0, 0, q);
#pragma unroll
    for (int q = 0; q < 8; ++q) dma(1, 1, q);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) dma(2, 2, q);
    __builtin_amdgcn_sched_barrier(0);
    sg_wait_vm<8>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int x = 0; x < 16; ++x) read_one(0, 0, x);
    for (int g = 0; g <= last; g += SG_GRP) {
#pragma unroll
        for (int i = 0; i < SG_GRP; ++i) {
            const int c = g + i, cn = c + 3 < last ? c + 3 : last;
            const int set = i & 1;
            // 64 MFMAs; after every second one half a fragment (one transpose read) of step c + 1, after every
            // eighth one load piece of step c + 3
#pragma unroll
            for (int x = 0; x < 16; ++x) {
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const int m = x * 4 + n, ia = m >> 3, jb = m & 7;
                    mfma_acc<T>(acc[ia][jb], fa[set][ia], fb[set][jb]);
                }
                read_one(set ^ 1, (i + 1) % SG_NS, x);
                if (x & 1) dma(cn, (i + 3) % SG_NS, x >> 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            sg_wait_vm<8>();
            __builtin_amdgcn_s_barrier();
        }
    }
    sg_wait_vm<0>();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last MFMAs leave the pipe before their accumulators are read
    __syncthreads();

    const int col_l = lane & 15, rgrp = (lane >> 4) * 4;
    if (a.ws) {
        // split K: the fp32 partial tile, 64 rows at a time through LDS (whole kilobyte row segments)
        constexpr int PITCH = 256 + 4;
        float *stage32 = reinterpret_cast<float *>(ring);
        float *W = a.ws + (int64_t)split * a.M * a.N;
#pragma unroll
        for (int slab = 0; slab < 4; ++slab) {               // rows 64 slab .. 64 slab + 63 of the tile
            if (wm == (slab >> 1)) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4)
#pragma unroll
                    for (int jb = 0; jb < 8; ++jb)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            stage32[(i4 * 16 + rgrp + r) * PITCH + wn * 128 + jb * 16 + col_l] = acc[(slab & 1) * 4 + i4][jb][r];
            }
            __syncthreads();
            for (int v = tid; v < 64 * 64; v += SG_THREADS) {
                const int rl = v >> 6, cv = v & 63;
                const int row = tm * 256 + slab * 64 + rl, col = tn * 256 + cv * 4;
                if (row < a.M && col < a.N)
                    *reinterpret_cast<v4f *>(&W[(int64_t)row * a.N + col]) = *reinterpret_cast<const v4f *>(&stage32[rl * PITCH + cv * 4]);
            }
            __syncthreads();
        }
        return;
    }
    // 16-bit result through LDS, written as whole 512-byte row segments
    T *stage = reinterpret_cast<T *>(ring);
#pragma unroll
    for (int ia = 0; ia < 8; ++ia)
#pragma unroll
        for (int jb = 0; jb < 8; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                stage[(wm * 128 + ia * 16 + rgrp + r) * SG_OLD + wn * 128 + jb * 16 + col_l] = Lp<T>::from_f(acc[ia][jb][r]);
    __syncthreads();
    T *C = reinterpret_cast<T *>(a.C);
#pragma unroll 4
    for (int v = tid; v < 256 * 32; v += SG_THREADS) {
        const int rl = v >> 5, cv = v & 31;
        const int row = tm * 256 + rl, col = tn * 256 + cv * 8;
        if (row >= a.M || col >= a.N) continue;
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

bool gemm_stream_tn_supported(int dtype, const BlockedGemmArgs &g) {
    if (dtype == LSTM_DTYPE_FP32) return false;
    if (!g.A.trans || !g.B.trans || !g.out_lp || g.accumulate || g.bias || g.batch > 1) return false;
    if (g.A.packed != g.B.packed) return false;
    if (g.M <= 0 || g.N <= 0 || g.K < 32 * SG_GRP || g.K % (32 * SG_GRP) != 0) return false;
    if (g.M % 8 != 0 || g.N % 8 != 0 || g.ldc % 8 != 0) return false;
    // split K: equal splits of whole groups of steps, partial sums in the caller's fp32 workspace
    if (g.splits > 1 && (!g.splitk_ws || (uintptr_t)g.splitk_ws % 16 || g.K % (32 * SG_GRP * g.splits) != 0)) return false;
    // 16-byte stores into C (a worker's row of a gradient matrix may start at any element: then the other kernel)
    if (!g.A.ptr || !g.B.ptr || !g.C || (uintptr_t)g.A.ptr % 16 || (uintptr_t)g.B.ptr % 16 || (uintptr_t)g.C % 16) return false;
    return g.A.ncb >= (g.M + 63) / 64 && g.B.ncb >= (g.N + 63) / 64;
}

int gemm_stream_tn(int dtype, const BlockedGemmArgs &g, hipStream_t stream) {
    if (!gemm_stream_tn_supported(dtype, g)) {
        set_error("gemm_stream_tn: unsupported product M=%d N=%d K=%d (16-bit result of 16-byte aligned blocked operands whose "
                  "rows are the contraction index, K a multiple of %d)", g.M, g.N, g.K, 32 * SG_GRP);
        return LSTM_ERR_INVALID;
    }
    StreamTnArgs a{};
    a.A = (const uint16_t *)g.A.ptr; a.B = (const uint16_t *)g.B.ptr; a.ncb_a = g.A.ncb; a.ncb_b = g.B.ncb;
    a.C = g.C; a.ldc = g.ldc; a.M = g.M; a.N = g.N; a.K = g.K;
    a.tiles_m = (g.M + 255) / 256; a.tiles_n = (g.N + 255) / 256;
    const int splits = g.splits > 1 ? g.splits : 1;
    a.ws = splits > 1 ? g.splitk_ws : nullptr;
    a.split_steps = g.K / 32 / splits;
    const double flops = 2.0 * g.M * g.N * g.K;
    const double bytes = 2.0 * ((double)g.M * g.K + (double)g.N * g.K + (double)g.M * g.N);
    KernelTimer timer(g.kclass, stream, flops, bytes);
    const dim3 grid(a.tiles_m * a.tiles_n * splits);
    if (g.A.packed) {
        if (dtype == LSTM_DTYPE_FP16) hipLaunchKernelGGL((gemm_stream_tn_kernel<_Float16, true>), grid, dim3(SG_THREADS), 0, stream, a);
        else hipLaunchKernelGGL((gemm_stream_tn_kernel<bf16_t, true>), grid, dim3(SG_THREADS), 0, stream, a);
    } else {
        if (dtype == LSTM_DTYPE_FP16) hipLaunchKernelGGL((gemm_stream_tn_kernel<_Float16, false>), grid, dim3(SG_THREADS), 0, stream, a);
        else hipLaunchKernelGGL((gemm_stream_tn_kernel<bf16_t, false>), grid, dim3(SG_THREADS), 0, stream, a);
    }
    LSTM_LAUNCH_CHECK();
    if (splits > 1) return splitk_reduce(dtype, g.splitk_ws, splits, g.M, g.N, g.C, g.ldc, stream);
    return LSTM_OK;
}

}  // namespace lstm
