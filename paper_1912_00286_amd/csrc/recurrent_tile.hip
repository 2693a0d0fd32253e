// Per-time-step kernels of the recurrence for wide layers (half / bfloat16 storage), several
// independent (layer, time) cells per launch.
//
// Forward : A_t = Ax_t + h_{t-1} U^T, gate non-linearities, cell and hidden update (fused).
// Backward: the recurrent data gradient dA_{t+1} U as four K-slices (one per gate), fp32 partials.
//
// Both are skinny GEMMs (M = batch) whose B operand, the 4H x H recurrent matrix, is read once per
// cell and never reused: a launch is bound by how fast the compute units can pull the operands in,
// not by the matrix pipes.  What this form does about it:
//   * a workgroup owns 32*MB batch rows x 128 B-operand rows over the whole K range of its product,
//     and wavefront w owns B block w (forward: gate w of 32 hidden units; backward: 32 of the 128
//     output units), so nothing is added up across wavefronts and the B fragments go from memory
//     straight into the registers the MFMA reads them from (packed operand layout, packed.h);
//   * the A operand (h_{t-1} or dA_{t+1}), which all four wavefronts need, is fetched ONCE per
//     workgroup, with direct-to-LDS loads into a ring of K chunks, and read from there;
//   * the workgroup needs 40-64 KB of LDS and at most 256 registers per lane, so several are resident per
//     compute unit, and a launch carries the cells of several layers (a layer runs a fixed number
//     of time steps behind the layer below it, see the schedule in api.hip): a launch then moves three
//     cells' bytes for one launch's ramp-up and tail;
//   * the four gates of a unit meet through the LDS ring's bytes once the product is done, in a
//     layout from which every thread finishes 8 consecutive units of one row with 16-byte accesses.
// Shapes: H a multiple of 128, batch a multiple of 32*MB (the host wrappers check).
#include "kernels.h"
#include "packed.h"

namespace lstm {
namespace {

typedef __attribute__((address_space(3))) void *lds_ptr;

// One K chunk of operands per ring stage; PF chunks are in flight ahead of the one being multiplied.
template <int MB> struct TileGeo {
    static constexpr int ROWS = 32 * MB;
    static constexpr int TILES = MB / 2;                 // packed A tiles (64 rows) per workgroup
    static constexpr int PF = MB == 4 ? 3 : 4;
    static constexpr int NS = PF + 1;
    static constexpr int STAGE_BYTES = TILES * A_CHUNK * 2;
    static constexpr int PIECES = TILES * 8 / 4;         // 1 KB pieces of a stage each wavefront fetches
    static constexpr int LDS_BYTES = NS * STAGE_BYTES;
    static_assert(LDS_BYTES >= 4 * ROWS * 32 * 4, "the gate exchange aliases the ring");
};

// s_waitcnt for the vector-memory counter alone: at most N of this wavefront's loads (register loads and
// direct-to-LDS loads alike) are still outstanding afterwards; they complete in issue order.
template <int N> __device__ __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// ... for the loads of k whole chunks (OPS loads each), k = 0 .. 3
template <int OPS> __device__ __forceinline__ void wait_vm_chunks(int k) {
    switch (k) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<OPS>(); break;
        case 2: wait_vm<2 * OPS>(); break;
        default: wait_vm<3 * OPS>(); break;
    }
}

// acc[mb] += A[32*MB rows, nch chunks] * B_w[32 rows, nch chunks]^T.
//   A0       : first packed chunk of the workgroup's first 64-row tile; tile t is a_tile_stride elements further
//   Bw       : first packed chunk of the B tile, already offset to this wavefront's block (+ wave * 64 fragments)
//   ring     : LDS, TileGeo<MB>::LDS_BYTES
//   NCH      : the number of chunks when known at compile time (the loop is then unrolled completely, which lets
//              the compiler count outstanding loads exactly), 0: `nch` chunks, known at run time
// Order inside a step: [wait until at most the loads of the chunks after c are outstanding: chunk c's A pieces and B
// fragments have landed] [barrier: every wavefront's share of chunk c is in LDS and everybody is done with chunk
// c - 1] [request chunk c + PF into the stage chunk c - 1 occupied] [multiply chunk c] [request the B fragments of
// chunk c + PF into the registers chunk c just left].  The requests of one chunk are issued between two consecutive
// barriers, which no instruction is moved across, so "the loads of the chunks after c" are the youngest ones.
template <typename T, int MB, int NCH>
__device__ __forceinline__ void tile_mainloop(const uint16_t *A0, int64_t a_tile_stride, const uint16_t *Bw, int nch_rt,
                                              unsigned char *ring, int wave, int lane, v16f (&acc)[MB]) {
    typedef TileGeo<MB> G;
    constexpr int PF = G::PF, NS = G::NS, OPS = G::PIECES + 4;
    static_assert(PF <= 4, "wait_vm_chunks covers up to three chunks in flight behind the current one");
    const int nch = NCH > 0 ? NCH : nch_rt;
    u32x4 breg[PF][4];
    auto issueA = [&](int c, int st) {
#pragma unroll
        for (int i = 0; i < G::PIECES; ++i) {
            const int g = wave * G::PIECES + i, tile = g >> 3, piece = g & 7;
            const u32x4 *src = reinterpret_cast<const u32x4 *>(A0 + tile * a_tile_stride + (int64_t)c * A_CHUNK) + piece * 64 + lane;
            __builtin_amdgcn_global_load_lds(src, (lds_ptr)(ring + st * G::STAGE_BYTES + g * 1024), 16, 0, 0);
        }
    };
    auto issueB = [&](u32x4 (&b)[4], int c) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(Bw + (int64_t)c * B_CHUNK) + lane;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) b[ks] = src[ks * 256];
    };
    // the A fragments of k-step ks + 1 travel from LDS while the MFMAs of k-step ks run; the scheduling groups
    // (0x100: LDS reads, 0x008: MFMAs) keep the compiler from putting every read right in front of its MFMA
    auto multiply = [&](const u32x4 (&b)[4], int st) {
        const u32x4 *L = reinterpret_cast<const u32x4 *>(ring + st * G::STAGE_BYTES) + lane;
        u32x4 af[2][MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) af[0][mb] = L[((mb >> 1) * 8 + (mb & 1)) * 64];
        __builtin_amdgcn_sched_group_barrier(0x100, MB, 0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) af[(ks + 1) & 1][mb] = L[((mb >> 1) * 8 + (ks + 1) * 2 + (mb & 1)) * 64];
                __builtin_amdgcn_sched_group_barrier(0x100, MB, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[mb] = Lp<T>::mfma(af[ks & 1][mb], b[ks], acc[mb]);
            __builtin_amdgcn_sched_group_barrier(0x008, MB, 0);
        }
    };
    auto step = [&](int c, u32x4 (&b)[4], int st, int stp) {
        const int behind = nch - 1 - c;                   // chunks requested after chunk c
        wait_vm_chunks<OPS>(behind < PF - 1 ? behind : PF - 1);
        __builtin_amdgcn_s_barrier();
        if (c + PF < nch) issueA(c + PF, stp);
        multiply(b, st);
        if (c + PF < nch) issueB(b, c + PF);
    };
    // The waits count loads from the youngest backwards, so the requests of one chunk have to be issued together, in
    // chunk order.  Between two barriers the steps below guarantee that; here, before the first barrier, the compiler
    // would interleave the loads of the PF chunks as it likes (it did: the second A piece of chunk 0 was issued
    // behind register loads of chunks 1 and 2, so the first step's wait did not cover it and a workgroup now and then
    // multiplied 32 rows of stale LDS bytes).  A scheduling fence after every chunk keeps the order.
#pragma unroll
    for (int i = 0; i < PF; ++i) {
        if (i < nch) { issueA(i, i); issueB(breg[i], i); }
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (NCH > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) step(c, breg[c % PF], c % NS, (c + PF) % NS);
    } else {
        int st = 0, stp = PF % NS;                        // stage of chunk c, stage chunk c + PF goes to
        for (int c = 0; c < nch; c += PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                if (c + i < nch) step(c + i, breg[i], st, stp);
                st = st + 1 == NS ? 0 : st + 1;
                stp = stp + 1 == NS ? 0 : stp + 1;
            }
        }
    }
}

template <int MB>
__device__ __forceinline__ void zero_acc(v16f (&acc)[MB]) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
}

// ---------------------------------------------------------------- forward
constexpr int TILE_MAX_CELLS = 4;
struct TileFwdCell {
    const void *hpk_prev;  // packed h_{t-1}: [n_mt][nkc] chunks of 64 x 64
    const void *Upk;       // packed U: [n_hb][nkc] chunks of 128 x 64, row block = gate
    const void *Ax;        // lp [B,4H]: input projection + bias of this step
    float *c_state;        // fp32 [B,H] in/out
    void *gates;           // lp [B,4H] out
    void *c_out, *h_out;   // lp [B,H] out (row-major); h_out may be null when only the packed / blocked copies are read
    void *hpk_next;        // packed h_t out
    void *h_blk;           // h_t out in 64x64 blocks (first block row of the time slot), or null
};
struct TileFwdArgs {
    TileFwdCell cell[TILE_MAX_CELLS];
    int B, H, nkc, blk_ncb, wgs_per_cell;
};

template <typename T, int MB, int NCH>
__global__ __launch_bounds__(256, 2) void lstm_tile_forward_kernel(TileFwdArgs a) {
    typedef TileGeo<MB> G;
    __shared__ __attribute__((aligned(1024))) unsigned char ring[G::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ci = blockIdx.x / a.wgs_per_cell;                     // uniform: the cell's argument block
    const TileFwdCell &c = a.cell[ci];
    const int lin = xcd_swizzle((int)blockIdx.x - ci * a.wgs_per_cell, a.wgs_per_cell);
    const int n_m2 = a.B / G::ROWS;
    const int mt2 = lin % n_m2, hb = lin / n_m2;                    // the row tiles of one unit block are neighbours
    const int H = a.H, G4 = 4 * a.H;
    v16f acc[MB];
    zero_acc<MB>(acc);
    tile_mainloop<T, MB, NCH>(reinterpret_cast<const uint16_t *>(c.hpk_prev) + (int64_t)mt2 * G::TILES * a.nkc * A_CHUNK, (int64_t)a.nkc * A_CHUNK,
                         reinterpret_cast<const uint16_t *>(c.Upk) + (int64_t)hb * a.nkc * B_CHUNK + wave * 64 * 8, a.nkc, ring, wave,
                         lane, acc);
    // the four gates of a unit meet: ex[gate][row][unit of the block], fp32, in the ring's bytes
    __syncthreads();                                                // every wavefront is done reading the ring
    float *ex = reinterpret_cast<float *>(ring);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            ex[(wave * G::ROWS + mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * 32 + (lane & 31)] = acc[mb][r];
    __syncthreads();
    // one item = 8 consecutive units of one row: 16-byte accesses throughout
    constexpr int ITEMS = G::ROWS * 4 / 256;
    const T *Ax = reinterpret_cast<const T *>(c.Ax);
    u32x4 vax[ITEMS][4];
    v4f vc[ITEMS][2];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int item = tid + 256 * it, rl = item >> 2, j8 = hb * 32 + (item & 3) * 8;
        const int64_t row = (int64_t)mt2 * G::ROWS + rl;
#pragma unroll
        for (int g = 0; g < 4; ++g) vax[it][g] = *reinterpret_cast<const u32x4 *>(Ax + row * G4 + g * H + j8);
        vc[it][0] = *reinterpret_cast<const v4f *>(c.c_state + row * H + j8);
        vc[it][1] = *reinterpret_cast<const v4f *>(c.c_state + row * H + j8 + 4);
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int item = tid + 256 * it, rl = item >> 2, ug = item & 3, j8 = hb * 32 + ug * 8;
        const int64_t row = (int64_t)mt2 * G::ROWS + rl;
        __attribute__((aligned(16))) float pre[4][8];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            *reinterpret_cast<v4f *>(pre[g]) = *reinterpret_cast<const v4f *>(ex + (g * G::ROWS + rl) * 32 + ug * 8);
            *reinterpret_cast<v4f *>(pre[g] + 4) = *reinterpret_cast<const v4f *>(ex + (g * G::ROWS + rl) * 32 + ug * 8 + 4);
        }
        __attribute__((aligned(16))) T ax[4][8], og[4][8], oc[8], oh[8];
        __attribute__((aligned(16))) float cn[8];
#pragma unroll
        for (int g = 0; g < 4; ++g) *reinterpret_cast<u32x4 *>(ax[g]) = vax[it][g];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float gi = sigmoidf_dev(pre[0][e] + Lp<T>::to_f(ax[0][e]));
            const float gf = sigmoidf_dev(pre[1][e] + Lp<T>::to_f(ax[1][e]));
            const float gg = tanhf_dev(pre[2][e] + Lp<T>::to_f(ax[2][e]));
            const float go = sigmoidf_dev(pre[3][e] + Lp<T>::to_f(ax[3][e]));
            const float cv = gf * vc[it][e >> 2][e & 3] + gi * gg;
            cn[e] = cv;
            og[0][e] = Lp<T>::from_f(gi); og[1][e] = Lp<T>::from_f(gf); og[2][e] = Lp<T>::from_f(gg); og[3][e] = Lp<T>::from_f(go);
            oc[e] = Lp<T>::from_f(cv);
            oh[e] = Lp<T>::from_f(go * tanhf_dev(cv));
        }
        T *gr = reinterpret_cast<T *>(c.gates) + row * G4 + j8;
#pragma unroll
        for (int g = 0; g < 4; ++g) *reinterpret_cast<u32x4 *>(gr + g * H) = *reinterpret_cast<const u32x4 *>(og[g]);
        *reinterpret_cast<v4f *>(c.c_state + row * H + j8) = *reinterpret_cast<const v4f *>(cn);
        *reinterpret_cast<v4f *>(c.c_state + row * H + j8 + 4) = *reinterpret_cast<const v4f *>(cn + 4);
        *reinterpret_cast<u32x4 *>(reinterpret_cast<T *>(c.c_out) + row * H + j8) = *reinterpret_cast<const u32x4 *>(oc);
        const u32x4 h8 = *reinterpret_cast<const u32x4 *>(oh);
        if (c.h_out) *reinterpret_cast<u32x4 *>(reinterpret_cast<T *>(c.h_out) + row * H + j8) = h8;
        // the next step's A operand: 8 units of a row are one 16-byte slot of the fragment order
        *reinterpret_cast<u32x4 *>(reinterpret_cast<T *>(c.hpk_next) + ((row >> 6) * a.nkc + (j8 >> 6)) * A_CHUNK +
                                   frag_offset((int)(row & 63), j8 & 63, 2)) = h8;
        if (c.h_blk)
            *reinterpret_cast<u32x4 *>(reinterpret_cast<T *>(c.h_blk) + ((row >> 6) * a.blk_ncb + (j8 >> 6)) * 4096 + (row & 63) * 64 + (j8 & 63)) = h8;
    }
}

// ---------------------------------------------------------------- backward product
constexpr int TILE_SLICES = 4;   // K-slices of the backward product: one gate each.  Two gates each (8 bytes of partial sums
                                 // per unit and direction instead of 16, half as many workgroups of twice the length) was
                                 // measured on the 3 x 2048-unit model: gate kernels 2.62 -> 2.46 ms per training step, step
                                 // kernels 10.3 -> 11.05 ms: slower in all
struct TileBwdCell {
    const void *dApk;      // packed dA_{t+1}: [n_mt][4][nkc] chunks of 64 x 64
    const void *UTpk;      // packed U^T: [n_nt][4][nkc] chunks of 128 x 64
    float *partials;       // fp32 [TILE_SLICES][B,H] out: one K-slice each
};
struct TileBwdArgs {
    TileBwdCell cell[TILE_MAX_CELLS];
    int B, H, nkc, wgs_per_cell;
};

// partial[q][b, j] = sum over the rows k of the gates of slice q of dA_next[b, k] * U[k, j]; the chunks of consecutive
// gates follow each other in both packed operands, so a slice is one run of NCH = (4 / TILE_SLICES) nkc chunks
template <typename T, int MB, int NCH>
__global__ __launch_bounds__(256, 2) void lstm_tile_backward_kernel(TileBwdArgs a) {
    typedef TileGeo<MB> G;
    __shared__ __attribute__((aligned(1024))) unsigned char ring[G::LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ci = blockIdx.x / a.wgs_per_cell;
    const TileBwdCell &c = a.cell[ci];
    const int lin = xcd_swizzle((int)blockIdx.x - ci * a.wgs_per_cell, a.wgs_per_cell);
    // slice major: the workgroups of one XCD share one K slice, so that XCD's L2 pulls only that
    // part of dA over the fabric
    constexpr int GPS = 4 / TILE_SLICES;                            // gates per slice
    const int per_q = a.wgs_per_cell / TILE_SLICES;
    const int q = lin / per_q, tile = lin - q * per_q;
    const int n_m2 = a.B / G::ROWS;
    const int mt2 = tile % n_m2, nt = tile / n_m2;
    v16f acc[MB];
    zero_acc<MB>(acc);
    tile_mainloop<T, MB, NCH>(reinterpret_cast<const uint16_t *>(c.dApk) + ((int64_t)mt2 * G::TILES * 4 + q * GPS) * a.nkc * A_CHUNK,
                         (int64_t)4 * a.nkc * A_CHUNK,
                         reinterpret_cast<const uint16_t *>(c.UTpk) + ((int64_t)nt * 4 + q * GPS) * a.nkc * B_CHUNK + wave * 64 * 8,
                         GPS * a.nkc, ring, wave, lane, acc);
    float *part = c.partials + (int64_t)q * a.B * a.H + (int64_t)mt2 * G::ROWS * a.H + nt * TN + wave * 32 + (lane & 31);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[(int64_t)(mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * a.H] = acc[mb][r];
}

#define LP_ONLY(dtype, T, ...)                                                       \
    if (dtype == LSTM_DTYPE_FP16) { using T = _Float16; __VA_ARGS__; }               \
    else if (dtype == LSTM_DTYPE_BF16) { using T = bf16_t; __VA_ARGS__; }            \
    else { set_error("recurrent kernels: dtype %d is not a 16-bit type", dtype); return LSTM_ERR_UNSUPPORTED; }

// Kernel instance by K chunks of a workgroup's product (`mult` runs of nkc chunks): the widths 1024 and 2048 get
// completely unrolled loops.
#define TILE_LAUNCH(T, MB_, kernel, mult, grid, s, a)                                                             \
    do {                                                                                                          \
        if ((a).nkc == 32) hipLaunchKernelGGL((kernel<T, MB_, 32 * (mult)>), grid, dim3(256), 0, s, a);            \
        else if ((a).nkc == 16) hipLaunchKernelGGL((kernel<T, MB_, 16 * (mult)>), grid, dim3(256), 0, s, a);       \
        else hipLaunchKernelGGL((kernel<T, MB_, 0>), grid, dim3(256), 0, s, a);                                    \
    } while (0)
#define TILE_DISPATCH(dtype, kernel, mult, grid, s, a) LP_ONLY(dtype, T, TILE_LAUNCH(T, TILE_MB, kernel, mult, grid, s, a))

// Rows per workgroup tile, in blocks of 32.  Measured on the 3 x 2048-unit model at batch 256 (three cells per
// launch): 64-row tiles 10.2 ms of step kernels per training step, 128-row tiles (a third fewer bytes into the
// compute units, but a third as many workgroups) 11.1 ms: the launches are bound by bytes from memory, which
// the tile height does not change, and the smaller tiles spread them more evenly.
constexpr int TILE_MB = 2;

}  // namespace

bool tile_kernels_supported(int dtype, int B, int H) {
    return dtype != LSTM_DTYPE_FP32 && H % 128 == 0 && B % 64 == 0 && B >= 64;
}
int tile_max_cells() { return TILE_MAX_CELLS; }
int tile_backward_slices() { return TILE_SLICES; }

int step_forward_tile(int dtype, const WaveCell *cells, int n_cells, int blk_ncb, int B, int H, hipStream_t s) {
    if (!tile_kernels_supported(dtype, B, H) || n_cells < 1 || n_cells > TILE_MAX_CELLS) {
        set_error("step_forward_tile: unsupported shape (B=%d, H=%d) or cell count %d", B, H, n_cells);
        return LSTM_ERR_UNSUPPORTED;
    }
    TileFwdArgs a;
    uintptr_t all = 0;
    for (int i = 0; i < TILE_MAX_CELLS; ++i) {
        const WaveCell &c = cells[i < n_cells ? i : 0];
        if (!c.hpk_prev || !c.Upk || !c.Ax || !c.c_state || !c.gates || !c.c_out || !c.hpk_next) {
            set_error("step_forward_tile: null operand in cell %d", i);
            return LSTM_ERR_INVALID;
        }
        all |= (uintptr_t)c.hpk_prev | (uintptr_t)c.Upk | (uintptr_t)c.Ax | (uintptr_t)c.c_state | (uintptr_t)c.gates | (uintptr_t)c.c_out |
               (uintptr_t)c.h_out | (uintptr_t)c.hpk_next | (uintptr_t)c.h_blk;
        a.cell[i] = TileFwdCell{c.hpk_prev, c.Upk, c.Ax, c.c_state, c.gates, c.c_out, c.h_out, c.hpk_next, c.h_blk};
    }
    if (all % 16 != 0) {
        set_error("step_forward_tile: operands must be 16-byte aligned");
        return LSTM_ERR_INVALID;
    }
    constexpr int mb = TILE_MB;
    a.B = B; a.H = H; a.nkc = H / SK; a.blk_ncb = blk_ncb; a.wgs_per_cell = (B / (32 * mb)) * (H / 32);
    // per cell: U read once; per unit the four pre-activations and c read, the four gates, c and h written
    const double bh = (double)B * H;
    KernelTimer timer(KC_GEMM_STEP, s, n_cells * 2.0 * B * 4.0 * H * H, n_cells * (2.0 * 4.0 * H * H + 26.0 * bh));
    const dim3 grid(a.wgs_per_cell * n_cells);
    TILE_DISPATCH(dtype, lstm_tile_forward_kernel, 1, grid, s, a);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int step_backward_gemm_tile(int dtype, const WaveGemm *g, int n, int B, int H, hipStream_t s) {
    if (!tile_kernels_supported(dtype, B, H) || n < 1 || n > TILE_MAX_CELLS) {
        set_error("step_backward_gemm_tile: unsupported shape (B=%d, H=%d) or product count %d", B, H, n);
        return LSTM_ERR_UNSUPPORTED;
    }
    TileBwdArgs a;
    for (int i = 0; i < TILE_MAX_CELLS; ++i) {
        const WaveGemm &c = g[i < n ? i : 0];
        if (!c.dApk || !c.Bpk || !c.partials || (((uintptr_t)c.dApk | (uintptr_t)c.Bpk | (uintptr_t)c.partials) % 16 != 0)) {
            set_error("step_backward_gemm_tile: null or misaligned operand in product %d", i);
            return LSTM_ERR_INVALID;
        }
        a.cell[i] = TileBwdCell{c.dApk, c.Bpk, c.partials};
    }
    constexpr int mb = TILE_MB;
    a.B = B; a.H = H; a.nkc = H / SK; a.wgs_per_cell = (B / (32 * mb)) * (H / TN) * TILE_SLICES;
    // per product: U and dA read once, one fp32 dh written
    KernelTimer timer(KC_GEMM_STEP, s, n * 2.0 * B * 4.0 * H * H, n * (2.0 * 4.0 * H * H + 12.0 * (double)B * H));
    const dim3 grid(a.wgs_per_cell * n);
    TILE_DISPATCH(dtype, lstm_tile_backward_kernel, 4 / TILE_SLICES, grid, s, a);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace lstm
