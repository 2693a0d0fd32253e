// Fused per-time-step kernels of the recurrence (half / bfloat16 storage).
//
// Forward:  A_t = Ax_t + h_{t-1} U^T, gate non-linearities, cell and hidden
//           update, all outputs written once.  One launch per step and layer.
// Backward: the recurrent data gradient dA_{t+1} U as four K-slices (one per
//           gate) written as fp32 partials; the BPTT gate kernel sums them.
//
// Both are skinny GEMMs (M = batch).  A workgroup owns 64 batch rows x 4 blocks
// of 32 B-operand rows (forward: the i,f,g,o rows of 32 hidden units, so the
// epilogue finds the four gates of a unit in one lane; backward: 128 hidden
// units) over a K range of at most H, and its 4 wavefronts split that K range
// four ways, so the K loop has no workgroup barrier; two chunks of global
// loads are kept in flight in registers.  The four partial accumulator sets are
// summed through LDS.
//
// These kernels are bound by how fast a compute unit can pull its operand
// slices out of L2 (measured: row-strided 128-byte reads reach about a fifth of
// what contiguous kilobyte reads do).  Since no operand element is shared
// between wavefronts, both operands are kept in MFMA-fragment order, packed
// and zero-padded: for every (tile, 64-wide K chunk) the 16 bytes each lane
// feeds to one MFMA are stored lane after lane, so a wavefront load instruction
// reads one contiguous kilobyte straight into the registers the MFMA consumes.
// No LDS staging, no bounds checks, no alignment assumption about the caller's
// tensors.  Block of one chunk: [k-step of 16][32-row block][lane][8 elements],
// lane = 32 * (k half) + row; 8 KB for the 64-row A operand, 16 KB for B.
//   U packed for the forward  : [hidden block of 32][K chunk] blocks, row block = gate
//   U packed for the backward : [unit tile of 128][gate][K chunk] blocks (transposed on the fly)
//   h / dA packed             : [batch tile of 64]([gate])[K chunk] blocks
// The epilogues write the next step's A operand directly in packed order (and
// in row-major / 64x64-blocked order for the whole-sequence GEMMs).
//
// Four families share those operands:
//   * the kernels above (any H; a second form, WIDE, for H <= 512 with >= 1024 rows);
//   * their multi-cell forms (several independent (layer, time) cells per launch) for the
//     anti-diagonal schedule of stacks of narrow layers;
//   * the narrow-layer kernels (H <= 768, H % 8 == 0): a whole cell per launch on 16x16 or 32x32
//     tiles, the BPTT cell with its products and gate arithmetic in ONE launch;
//   * the row-ownership kernels (H <= 256, from 3072 rows per step: stacked workers): a layer's whole
//     recurrence in ONE launch per direction, a workgroup walking its 32 rows through all time steps.
// The host wrappers at the end of the file pick the family from the shape.
#include "kernels.h"
#include "packed.h"

namespace lstm {
namespace {

// TM, NBLK, TN, SK, A_CHUNK, B_CHUNK, frag_offset, xcd_swizzle: packed.h
constexpr int NLD_A = TM * SK / 8 / 64;   // 16-byte loads per lane and chunk, A operand (8)
constexpr int NLD_B = TN * SK / 8 / 64;   // same, B operand (16)
constexpr int RED_FLOATS = 8 * 16 * 64;   // one wavefront's 8 accumulator blocks

// A small kernel in a chain of dependent launches starts with dependent memory round trips (arguments,
// then operands), and the compiler fetches kernel arguments lazily, next to their first use: up to nine
// scalar loads one after the other were measured.  Naming a value as an input of an empty asm statement
// makes its load issue there, together with its neighbours'.
template <typename V>
__device__ __forceinline__ void fetch_now(const V &v) { asm volatile("" ::"s"(v)); }

__device__ __forceinline__ void load_chunk(u32x4 (&ra)[NLD_A], u32x4 (&rb)[NLD_B], const u32x4 *a, const u32x4 *b, int lane) {
#pragma unroll
    for (int i = 0; i < NLD_A; ++i) ra[i] = a[lane + 64 * i];
#pragma unroll
    for (int i = 0; i < NLD_B; ++i) rb[i] = b[lane + 64 * i];
}

template <typename T>
__device__ __forceinline__ void mfma_chunk(const u32x4 (&ra)[NLD_A], const u32x4 (&rb)[NLD_B], v16f (&acc)[2][NBLK]) {
#pragma unroll
    for (int ks = 0; ks < SK / 16; ++ks)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb) acc[mb][nb] = Lp<T>::mfma(ra[ks * 2 + mb], rb[ks * NBLK + nb], acc[mb][nb]);
}

// acc[mb][nb] += sum over chunks c in [c0, c1) of Apk[c] * Bpk[c]^T with both
// operands in fragment order.  `rot` rotates the order in which the chunks are
// visited.  Two register sets: while one chunk feeds the MFMAs the next one is
// already loaded and the one after is in flight.
template <typename T>
__device__ __forceinline__ void packed_mainloop(const uint16_t *Apk, const uint16_t *Bpk, int c0, int c1, int rot, int lane,
                                                v16f (&acc)[2][NBLK], const uint16_t *Apk2 = nullptr,
                                                const uint16_t *Bpk2 = nullptr, int nkc1 = 0) {
    // With a second operand pair the chunk list is the concatenation [pair 1: nkc1 chunks][pair 2],
    // so the load pipeline runs across the boundary between the two products.
    const int nst = c1 - c0;
    if (nst <= 0) return;
    rot %= nst;
    auto pa = [&](int s) {
        int ss = s + rot;
        if (ss >= nst) ss -= nst;
        const int c = c0 + ss;
        return reinterpret_cast<const u32x4 *>(Apk2 && c >= nkc1 ? Apk2 + (int64_t)(c - nkc1) * A_CHUNK : Apk + (int64_t)c * A_CHUNK);
    };
    auto pb = [&](int s) {
        int ss = s + rot;
        if (ss >= nst) ss -= nst;
        const int c = c0 + ss;
        return reinterpret_cast<const u32x4 *>(Bpk2 && c >= nkc1 ? Bpk2 + (int64_t)(c - nkc1) * B_CHUNK : Bpk + (int64_t)c * B_CHUNK);
    };
    u32x4 ra0[NLD_A], rb0[NLD_B], ra1[NLD_A], rb1[NLD_B];
    load_chunk(ra0, rb0, pa(0), pb(0), lane);
    if (nst > 1) load_chunk(ra1, rb1, pa(1), pb(1), lane);
    int s = 0;
    for (; s + 4 <= nst; s += 2) {           // branch-free body: both refills are in range
        mfma_chunk<T>(ra0, rb0, acc);
        load_chunk(ra0, rb0, pa(s + 2), pb(s + 2), lane);
        mfma_chunk<T>(ra1, rb1, acc);
        load_chunk(ra1, rb1, pa(s + 3), pb(s + 3), lane);
    }
    // tail: 1, 2 or 3 chunks left, set 0 holds chunk s, set 1 chunk s + 1
    mfma_chunk<T>(ra0, rb0, acc);
    if (s + 2 < nst) load_chunk(ra0, rb0, pa(s + 2), pb(s + 2), lane);
    if (s + 1 < nst) mfma_chunk<T>(ra1, rb1, acc);
    if (s + 2 < nst) mfma_chunk<T>(ra0, rb0, acc);
}

// Sum the four wavefronts' accumulators through LDS.  On return wavefront q
// holds in out[rr][nb] (rr = 0..7) the totals for m-block (q >> 1), accumulator
// registers r = 8 (q & 1) + rr, B block nb.
__device__ __forceinline__ void reduce_waves(float *red, int wave, int lane, v16f (&acc)[2][NBLK], float (&out)[8][NBLK]) {
    // four consecutive accumulator registers travel as one 16-byte LDS access
    v4f *red4 = reinterpret_cast<v4f *>(red);
    v4f *mine = red4 + wave * (RED_FLOATS / 4);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                v4f v = {acc[mb][nb][4 * r4], acc[mb][nb][4 * r4 + 1], acc[mb][nb][4 * r4 + 2], acc[mb][nb][4 * r4 + 3]};
                mine[((mb * NBLK + nb) * 4 + r4) * 64 + lane] = v;
            }
    __syncthreads();
    const int mb = wave >> 1, rq = (wave & 1) * 2;
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int nb = 0; nb < NBLK; ++nb) {
            const int idx = ((mb * NBLK + nb) * 4 + rq + q) * 64 + lane;
            const v4f s = (red4[idx] + red4[RED_FLOATS / 4 + idx]) + (red4[2 * (RED_FLOATS / 4) + idx] + red4[3 * (RED_FLOATS / 4) + idx]);
#pragma unroll
            for (int k = 0; k < 4; ++k) out[q * 4 + k][nb] = s[k];
        }
}

__device__ __forceinline__ void zero_acc(v16f (&acc)[2][NBLK]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
}

// ---------------------------------------------------------------- forward
struct FwdArgs {
    const void *hpk_prev;  // packed h_{t-1}: [n_mt][nkc][64][64]
    const void *Upk;       // packed U: [n_hb][nkc][128][64]
    const void *Ax;        // lp [B,4H], input projection + bias of this step; null: computed here from xpk, Wpk, bias
    const void *xpk;       // packed input of this step (the layer below's h_t), same layout as hpk_prev
    const void *Wpk;       // packed W, same layout as Upk (input width = H)
    const void *bias;      // lp [4H]
    float *c_state;        // fp32 [B,H] in/out
    void *gates;           // lp [B,4H] out
    void *c_out;           // lp [B,H] out
    void *h_out;           // lp [B,H] out (row-major)
    void *hpk_next;        // packed h_t out
    void *h_blk;           // h_t out in 64x64 blocks (first block row of this time slot), or null
    int blk_ncb;           // column blocks per row block of h_blk
    int B, H, n_mt, nkc;
    int nkc2;              // K chunks of the input projection done here (xpk / Wpk), when Ax is null
};

// WIDE = false: the four wavefronts split the K range of one 64-row tile and their partial
//                accumulators are summed through LDS (large H: operand bytes per CU are what counts).
// WIDE = true : workgroups of one wavefront, each with a 64-row tile of its own over the whole K
//                range; no LDS, no reduction (small H with many batch rows, where the reduction
//                would cost more than the product); several such wavefronts share a SIMD and
//                hide each other's latencies.
template <typename T, bool WIDE>
__device__ __forceinline__ void forward_cell(const FwdArgs &a, int tile, int rot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = tile % a.n_mt, hb = tile / a.n_mt;
    const int m0 = mt * TM, j0 = hb * 32;
    const int H = a.H, G = 4 * a.H;
    // K chunks of this cell: the recurrent product, then (a cell that projects its own input) the
    // layer below's h_t times W^T; the wavefronts split the whole list
    const int nch = a.Ax ? a.nkc : a.nkc + a.nkc2;
    const int cpw = (nch + 3) / 4;                         // chunks per wavefront
    const int c0 = WIDE ? 0 : min(nch, wave * cpw), c1 = WIDE ? nch : min(nch, c0 + cpw);
    v16f acc[2][NBLK];
    zero_acc(acc);
    packed_mainloop<T>(reinterpret_cast<const uint16_t *>(a.hpk_prev) + (int64_t)mt * a.nkc * A_CHUNK,
                       reinterpret_cast<const uint16_t *>(a.Upk) + (int64_t)hb * a.nkc * B_CHUNK, c0, c1, rot, lane, acc,
                       a.Ax ? nullptr : reinterpret_cast<const uint16_t *>(a.xpk) + (int64_t)mt * a.nkc2 * A_CHUNK,
                       a.Ax ? nullptr : reinterpret_cast<const uint16_t *>(a.Wpk) + (int64_t)hb * a.nkc2 * B_CHUNK, a.nkc);
    const int j = j0 + (lane & 31);
    const int jc = min(j, H - 1);
    T *gates = reinterpret_cast<T *>(a.gates);
    T *c_out = reinterpret_cast<T *>(a.c_out);
    T *h_out = reinterpret_cast<T *>(a.h_out);
    T *hpk = reinterpret_cast<T *>(a.hpk_next) + ((int64_t)mt * a.nkc + (min(j, a.nkc * SK - 1) >> 6)) * A_CHUNK;
    // The step's input projection and the previous cell state do not depend on the GEMM: a
    // group of 8 accumulator rows requests them first (addresses clamped into the tensors;
    // out-of-range lanes never store) and consumes them after the pre-activations are ready.
    auto load_group = [&](int mb, int rh, float (&axv)[8][4], float (&cprev)[8]) {
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int r = rh + rr;
            const int row = min(m0 + mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), a.B - 1);
            // with the projection done above only the bias is left to add
            const T *ax = a.Ax ? reinterpret_cast<const T *>(a.Ax) + (int64_t)row * G + jc : reinterpret_cast<const T *>(a.bias) + jc;
#pragma unroll
            for (int g = 0; g < 4; ++g) axv[rr][g] = Lp<T>::to_f(ax[g * H]);
            cprev[rr] = a.c_state[(int64_t)row * H + jc];
        }
    };
    auto finish_group = [&](int mb, int rh, const float (&pre)[8][NBLK], const float (&axv)[8][4], const float (&cprev)[8]) {
        if (j0 + 32 >= H && j0 + 32 < a.nkc * SK) {
            // the last block of 32 units ends in the first half of a 64-column chunk: nobody owns the second
            // half, so this workgroup clears it (column j + 32 lies in the same chunk as column j)
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const int r = rh + rr;
                const int rl = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (m0 + rl < a.B) hpk[frag_offset(rl, (j & 63) + 32, 2)] = Lp<T>::from_f(0.0f);
            }
        }
        if (j >= H) {
            // padding columns of the packed h_t inside this block of 32 are written as zeros (with the half
            // chunk above: every column up to the next multiple of 64), so that a slot never touched before can
            // serve as the next step's operand
            if (j < a.nkc * SK) {
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int r = rh + rr;
                    const int rl = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                    if (m0 + rl < a.B) hpk[frag_offset(rl, j & 63, 2)] = Lp<T>::from_f(0.0f);
                }
            }
            return;
        }
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int r = rh + rr;
            const int rl = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            const int row = m0 + rl;
            const float gi = sigmoidf_dev(pre[rr][0] + axv[rr][0]);
            const float gf = sigmoidf_dev(pre[rr][1] + axv[rr][1]);
            const float gg = tanhf_dev(pre[rr][2] + axv[rr][2]);
            const float go = sigmoidf_dev(pre[rr][3] + axv[rr][3]);
            const float c = gf * cprev[rr] + gi * gg;
            const T h = Lp<T>::from_f(go * tanhf_dev(c));
            if (row >= a.B) continue;
            const int64_t e = (int64_t)row * H + j;
            a.c_state[e] = c;
            T *gr = gates + (int64_t)row * G + j;
            gr[0] = Lp<T>::from_f(gi);
            gr[H] = Lp<T>::from_f(gf);
            gr[2 * H] = Lp<T>::from_f(gg);
            gr[3 * H] = Lp<T>::from_f(go);
            c_out[e] = Lp<T>::from_f(c);
            h_out[e] = h;
            hpk[frag_offset(rl, j & 63, 2)] = h;
            if (a.h_blk)
                reinterpret_cast<T *>(a.h_blk)[((int64_t)(row >> 6) * a.blk_ncb + (j >> 6)) * 4096 + (row & 63) * 64 + (j & 63)] = h;
        }
    };
    if constexpr (WIDE) {
        // four groups of 8 accumulator rows; the loads of the next group are in flight while
        // the current one is finished
        float axv[2][8][4], cprev[2][8];
        load_group(0, 0, axv[0], cprev[0]);
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int mb = grp >> 1, rh = (grp & 1) * 8;
            if (grp < 3) load_group((grp + 1) >> 1, ((grp + 1) & 1) * 8, axv[(grp + 1) & 1], cprev[(grp + 1) & 1]);
            float pre[8][NBLK];
#pragma unroll
            for (int rr = 0; rr < 8; ++rr)
#pragma unroll
                for (int nb = 0; nb < NBLK; ++nb) pre[rr][nb] = acc[mb][nb][rh + rr];
            finish_group(mb, rh, pre, axv[grp & 1], cprev[grp & 1]);
        }
    } else {
        __shared__ __attribute__((aligned(16))) float smem[4 * RED_FLOATS];   // 128 KB: cross-wavefront reduction
        const int mb = wave >> 1, rh = (wave & 1) * 8;
        float axv[8][4], cprev[8], pre[8][NBLK];
        load_group(mb, rh, axv, cprev);                    // in flight during the reduction
        reduce_waves(smem, wave, lane, acc, pre);
        finish_group(mb, rh, pre, axv, cprev);
    }
}

template <typename T, bool WIDE>
__global__ __launch_bounds__(256) void lstm_step_forward_kernel(FwdArgs a) {
    forward_cell<T, WIDE>(a, xcd_swizzle(blockIdx.x, gridDim.x), (int)blockIdx.x);
}

// Several independent cells in one launch: layer l at time t depends on (l, t-1) and (l-1, t),
// so the cells of one anti-diagonal l + t = d can run together.  Stacks of narrow layers are
// bound by the chain of dependent launches (T * L of them layer by layer); along the diagonals
// the chain is T + L - 1 long and each launch carries up to L cells' workgroups.
constexpr int WAVE_MAX_CELLS = 8;
struct WaveFwdArgs {
    FwdArgs cell[WAVE_MAX_CELLS];
    int wgs_per_cell;
};
template <typename T>
__global__ __launch_bounds__(256) void lstm_wave_forward_kernel(WaveFwdArgs w) {
    const int c = blockIdx.x / w.wgs_per_cell;             // uniform: selects the cell's argument block
    forward_cell<T, false>(w.cell[c], (int)blockIdx.x - c * w.wgs_per_cell, (int)blockIdx.x);
}

// ---------------------------------------------------------------- a layer's whole forward recurrence in one launch
// Batch rows never interact, so a workgroup that owns 32 rows and ALL hidden units can walk them through the T
// time steps on its own: no launch per step and nothing crosses workgroups.  Per step it contracts its rows of
// h_{t-1} (kept in LDS in fragment order, written by its own epilogue one step earlier) with the packed U and its
// rows of x_t (packed input sequence, fetched into LDS one step ahead) with the packed W, one block of 32 units x
// 4 gates per wavefront (eight wavefronts), keeps c_t in registers in the accumulator layout, and writes the saved
// gates, c_t, h_t (row-major, packed for the layer above, blocked for the weight-gradient GEMMs) as it goes.
// Workgroups drift apart in time, so the products of one run under the stores of another, which the lock-step
// grid of a per-step launch cannot do.  U and W stream from L2 every step (the half chunks of K that are all
// padding are skipped; the first fragments of the next step are requested before the epilogue).  Used with
// thousands of rows per step (stacked workers) and H <= 256.
struct RowsFwdArgs {
    const void *hseq;      // packed h slots [T+1][n_mt][nkc][64][64]: slot 0 = h_0 (in), slot t + 1 = h_t (out)
    const void *xseq;      // packed input slots [T][n_mt][nkc2][64][64]
    int64_t slot_h, slot_x;   // elements per slot
    const void *Upk, *Wpk, *bias;
    float *c_state;        // fp32 [B,H]: c_0 in, c_T out
    void *gates;           // lp [T][B,4H] out
    void *c_out, *h_out;   // lp [B,H] of step 0 (slot 1 of the saved sequences), the steps follow at B*H
    void *h_blk;           // blocked h of step 0 (slot 1), or null
    int64_t slot_blk;      // elements per time slot of h_blk
    int blk_ncb, T, B, H, nkc, nkc2;
    int in_width;          // columns of x (the rest of its last chunk is zero padding and is skipped)
    int all_h_out;         // 0: only h_T goes to h_out (a layer whose row-major h_t nobody reads)
    int write_hpk;         // 0: the packed h_t slots are not written (no layer above reads them)
};
template <typename T>
__global__ __launch_bounds__(512) void lstm_rows_forward_kernel(RowsFwdArgs a) {
    constexpr int HCH = 32 * SK;                       // elements of a 32-row chunk in LDS: [ks][lane][8]
    constexpr int STAGE_LD = 40;                       // elements per row of a staging tile (80 bytes: 16-byte aligned, off the bank stride)
    // both operands' rows for one step, in fragment order: chunks [0, nkc) = h_{t-1}, [nkc, nkc + nkc2) = x_t
    __shared__ __attribute__((aligned(16))) uint16_t abuf[2][8 * HCH];
    __shared__ __attribute__((aligned(16))) T stage[8][32 * STAGE_LD];
    const int tid = threadIdx.x, lane = tid & 63;
    const int hb = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront = block of 32 units x 4 gates
    const int mt = blockIdx.x >> 1, mb = blockIdx.x & 1;
    const int r0 = mt * TM + mb * 32;
    if (r0 >= a.B) return;                             // the second half of a ragged last tile
    const int H = a.H, G = 4 * a.H, n_hb = (H + 31) / 32;
    // half chunks (two k-steps of 16) of the step's two products; all-padding halves at the end of K are left out
    const int nqh = (H + 31) / 32, nq = nqh + (a.in_width + 31) / 32;
    // chunk c, k-step ks of these rows is fragment (c*8 + ks*2 + mb) of the packed 64-row tile
    auto tile_frag = [&](int v) { return ((v >> 8) * 8 + ((v >> 6) & 3) * 2 + mb) * 64 + (v & 63); };
    const u32x4 *xsrc = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.xseq) + (int64_t)mt * a.nkc2 * A_CHUNK);
    const int64_t xstep = a.slot_x / 8;                // 16-byte units per input slot
    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(reinterpret_cast<const uint16_t *>(a.hseq) + (int64_t)mt * a.nkc * A_CHUNK);
        u32x4 *dst = reinterpret_cast<u32x4 *>(abuf[0]);
        for (int v = tid; v < a.nkc * 256; v += 512) dst[v] = src[tile_frag(v)];
        for (int v = tid; v < a.nkc2 * 256; v += 512) dst[a.nkc * 256 + v] = xsrc[tile_frag(v)];
    }
    const bool active = hb < n_hb;                     // uniform over the wavefront
    const int col = lane & 31, rsub = (lane >> 5) * 4;
    const int j = hb * 32 + col, jc = min(j, H - 1);
    float creg[16], breg[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) breg[g] = Lp<T>::to_f(reinterpret_cast<const T *>(a.bias)[g * H + jc]);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = min(r0 + (r >> 2) * 8 + rsub + (r & 3), a.B - 1);
        creg[r] = a.c_state[(int64_t)row * H + jc];
    }
    __syncthreads();
    const int hbc = min(hb, n_hb - 1);
    const uint16_t *Upk = reinterpret_cast<const uint16_t *>(a.Upk) + (int64_t)hbc * a.nkc * B_CHUNK;
    const uint16_t *Wpk = reinterpret_cast<const uint16_t *>(a.Wpk) + (int64_t)hbc * a.nkc2 * B_CHUNK;
    const bool pad_half = hb * 32 + 32 >= H && hb * 32 + 32 < a.nkc * SK;   // nobody owns the chunk's second half
    // the weights of a half chunk: eight 16-byte fragments per lane (two k-steps x four gates)
    auto loadB = [&](u32x4 (&rb)[8], int q) {
        const bool rec = q < nqh;
        const int q2 = rec ? q : q - nqh;
        const u32x4 *b = reinterpret_cast<const u32x4 *>((rec ? Upk : Wpk) + (int64_t)(q2 >> 1) * B_CHUNK) + (q2 & 1) * 512;
#pragma unroll
        for (int i = 0; i < 8; ++i) rb[i] = b[lane + 64 * i];
    };
    u32x4 rb0[8], rb1[8];
    loadB(rb0, 0);
    loadB(rb1, 1);                                     // nq >= 2: at least one half chunk per product
    for (int t = 0; t < a.T; ++t) {
        // x_{t+1} of these rows is requested now and put into the other buffer at the end of the step
        u32x4 xnext[2];
        const bool more = t + 1 < a.T;
        if (more) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int v = tid + 512 * i;
                if (v < a.nkc2 * 256) xnext[i] = xsrc[(int64_t)(t + 1) * xstep + tile_frag(v)];
            }
        }
        T *hN = reinterpret_cast<T *>(abuf[(t + 1) & 1]);
        if (active) {
            const u32x4 *A = reinterpret_cast<const u32x4 *>(abuf[t & 1]);
            v16f acc[NBLK];
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[nb][r] = 0.0f;
            // half-chunk list: the recurrent product (h, U), then the input projection (x, W)
            auto loadA = [&](u32x4 (&ra)[2], int q) {
                const bool rec = q < nqh;
                const int q2 = rec ? q : q - nqh, ca = (rec ? 0 : a.nkc) + (q2 >> 1), hf = q2 & 1;
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) ra[k2] = A[(ca * 4 + hf * 2 + k2) * 64 + lane];
            };
            auto mm = [&](const u32x4 (&ra)[2], const u32x4 (&rb)[8]) {
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
                    for (int nb = 0; nb < NBLK; ++nb) acc[nb] = Lp<T>::mfma(ra[k2], rb[k2 * NBLK + nb], acc[nb]);
            };
            u32x4 ra0[2], ra1[2];
            loadA(ra0, 0);                             // the weights of half chunks 0 and 1 are already in rb0 / rb1
            loadA(ra1, 1);
            int s = 0;
            for (; s + 4 <= nq; s += 2) {              // branch-free body: both refills are in range
                mm(ra0, rb0);
                loadB(rb0, s + 2); loadA(ra0, s + 2);
                mm(ra1, rb1);
                loadB(rb1, s + 3); loadA(ra1, s + 3);
            }
            // tail: two or three half chunks left, set 0 holds s, set 1 holds s + 1
            mm(ra0, rb0);
            if (s + 2 < nq) { loadB(rb0, s + 2); loadA(ra0, s + 2); }
            mm(ra1, rb1);
            loadB(rb1, 1);                             // the next step's first weights travel during this step's epilogue
            if (s + 2 < nq) mm(ra0, rb0);
            loadB(rb0, 0);
            // Gate arithmetic in the accumulator layout (this lane: the four gates of unit j for 16 rows), then
            // every output goes through the wavefront's 32 x 32 staging tile in LDS, so that a lane stores 8
            // consecutive units of one row (16 bytes) instead of one unit of sixteen rows: a sixteenth of the
            // store instructions.  The tile is private to the wavefront, whose LDS accesses execute in
            // program order: no barrier between writing it in one layout and reading it in the other.
            T *tile = stage[hb];
            T *tw = tile + rsub * STAGE_LD + col;                  // + crow * STAGE_LD: element (row, unit) of the tile
            const int irow = lane >> 2, igrp = (lane & 3) * 8;     // item k of this lane: row irow + 16 k, units igrp..
            const int j8 = hb * 32 + igrp;
            const bool units8 = j8 < H;                            // H % 8 == 0: a group of 8 is inside or outside
            const bool pad8 = !units8 && j8 < a.nkc * SK;          // padding columns of the packed operand
            float gv[4][16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                gv[0][r] = sigmoidf_dev(acc[0][r] + breg[0]);
                gv[1][r] = sigmoidf_dev(acc[1][r] + breg[1]);
                gv[2][r] = tanhf_dev(acc[2][r] + breg[2]);
                gv[3][r] = sigmoidf_dev(acc[3][r] + breg[3]);
                creg[r] = gv[1][r] * creg[r] + gv[0][r] * gv[2][r];
            }
            auto exchange = [&](const float (&v)[16], u32x4 (&out)[2]) {
#pragma unroll
                for (int r = 0; r < 16; ++r) tw[((r >> 2) * 8 + (r & 3)) * STAGE_LD] = Lp<T>::from_f(v[r]);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int k = 0; k < 2; ++k) out[k] = *reinterpret_cast<const u32x4 *>(tile + (irow + 16 * k) * STAGE_LD + igrp);
                __builtin_amdgcn_wave_barrier();
            };
            u32x4 o8[2];
            const int kc8 = j8 >> 6, kk8 = j8 & 63;
            T *gates = reinterpret_cast<T *>(a.gates) + (int64_t)t * a.B * G + j8;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                exchange(gv[g], o8);
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int row = r0 + irow + 16 * k;
                    if (units8 && row < a.B) *reinterpret_cast<u32x4 *>(gates + (int64_t)row * G + g * H) = o8[k];
                }
            }
            float hv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) hv[r] = gv[3][r] * tanhf_dev(creg[r]);
            exchange(creg, o8);
            T *c_out = reinterpret_cast<T *>(a.c_out) + (int64_t)t * a.B * H + j8;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int row = r0 + irow + 16 * k;
                if (units8 && row < a.B) *reinterpret_cast<u32x4 *>(c_out + (int64_t)row * H) = o8[k];
            }
            exchange(hv, o8);
            T *h_out = reinterpret_cast<T *>(a.h_out) + (int64_t)t * a.B * H + j8;
            T *hpk = const_cast<T *>(reinterpret_cast<const T *>(a.hseq)) + (int64_t)(t + 1) * a.slot_h + ((int64_t)mt * a.nkc + kc8) * A_CHUNK;
            T *h_blk = a.h_blk ? reinterpret_cast<T *>(a.h_blk) + (int64_t)t * a.slot_blk + ((int64_t)mt * a.blk_ncb + kc8) * 4096 + kk8 : nullptr;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int rl = irow + 16 * k, row = r0 + rl;
                const u32x4 h8 = units8 ? o8[k] : u32x4{0u, 0u, 0u, 0u};
                // next step's operand: 8 units of a row are one 16-byte slot of the fragment order (zero in the padding)
                const int slot32 = ((kc8 * 4 + (kk8 >> 4)) * 64 + ((kk8 >> 3) & 1) * 32 + rl) * 8;
                if (units8 || pad8) *reinterpret_cast<u32x4 *>(hN + slot32) = h8;
                if (pad_half) *reinterpret_cast<u32x4 *>(hN + slot32 + 2 * 512) = u32x4{0u, 0u, 0u, 0u};   // columns + 32: nobody owns them
                if (row >= a.B) continue;
                if (a.write_hpk) {
                    if (units8 || pad8) *reinterpret_cast<u32x4 *>(hpk + frag_offset(mb * 32 + rl, kk8, 2)) = h8;
                    if (pad_half) *reinterpret_cast<u32x4 *>(hpk + frag_offset(mb * 32 + rl, kk8 + 32, 2)) = u32x4{0u, 0u, 0u, 0u};
                }
                if (!units8) continue;
                if (a.all_h_out || !more) *reinterpret_cast<u32x4 *>(h_out + (int64_t)row * H) = h8;
                if (h_blk) *reinterpret_cast<u32x4 *>(h_blk + (mb * 32 + rl) * 64) = h8;
            }
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int v = tid + 512 * i;
                if (v < a.nkc2 * 256) reinterpret_cast<u32x4 *>(hN)[a.nkc * 256 + v] = xnext[i];
            }
        }
        __syncthreads();                               // h_t of every unit block and x_{t+1} are in LDS before the next step reads them
    }
    if (active && j < H) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = r0 + (r >> 2) * 8 + rsub + (r & 3);
            if (row < a.B) a.c_state[(int64_t)row * H + j] = creg[r];
        }
    }
}

// ---------------------------------------------------------------- a layer's whole BPTT recurrence in one launch
// The same ownership backwards: a workgroup walks its 32 rows from t = T-1 down to 0.  dA_{t+1} of its rows (all
// four gates) sits in LDS in fragment order; wavefront w contracts it with the packed U^T for its block of 32
// units (all 4H gate rows: nothing to add up across wavefronts), turns the 32 x 32 result round through its
// staging tile so that a lane holds 8 consecutive units of two rows, and does the gate arithmetic there: the saved
// gates, c_t, c_{t-1} and the gradient from above arrive as 16-byte loads requested before the product, dA_t
// leaves as 16-byte stores (LDS for the next step, the blocked and / or row-major copy for the whole-sequence
// GEMMs), the cell-state gradient never leaves the registers.
struct RowsBwdArgs {
    const void *UTpk;      // packed U^T: [n_nt][4][nkc][128][64]
    const void *dh_above;  // lp [T][B,H]
    const void *gates;     // lp [T][B,4H]
    const void *cs;        // lp [T+1][B,H]: c_{t-1} is slot t, c_t slot t + 1
    void *dA;              // lp [T][B,4H] row-major, or null
    void *dAblk;           // dA in 64x64 blocks, slot_blk elements per time step, or null
    int64_t slot_blk;
    float *bias_partial;   // [gridDim.x][4H] out or null: column sums of this workgroup's dA rows over all steps
    int blk_ncb, T, B, H, nkc;
};
template <typename T>
__global__ __launch_bounds__(512) void lstm_rows_backward_kernel(RowsBwdArgs a) {
    constexpr int HCH = 32 * SK;                       // elements of a 32-row chunk in LDS: [ks][lane][8]
    constexpr int SLD = 36;                            // floats per row of a staging tile
    __shared__ __attribute__((aligned(16))) uint16_t dabuf[16 * HCH];      // [gate][nkc <= 4] chunks
    __shared__ __attribute__((aligned(16))) float stage[8][32 * SLD];
    // the cell-state gradient of a lane's 2 x 8 units: private, but kept in LDS (four 16-byte slots per lane) so that
    // the registers can hold the bias gradient's running sums instead
    __shared__ __attribute__((aligned(16))) v4f dcl[4][512];
    const int tid = threadIdx.x, lane = tid & 63;
    const int hb = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront = block of 32 units
    const int mt = blockIdx.x >> 1, mb = blockIdx.x & 1;
    const int r0 = mt * TM + mb * 32;
    if (r0 >= a.B) {                                   // (an odd group past the last row: its sums are zero)
        if (a.bias_partial)
            for (int c = tid; c < 4 * a.H; c += 512) a.bias_partial[(int64_t)blockIdx.x * 4 * a.H + c] = 0.0f;
        return;
    }
    const int H = a.H, G = 4 * a.H, n_hb = (H + 31) / 32;
    const int nq = 4 * n_hb;                           // half chunks of the contraction: gate = q % 4, half chunk q / 4
    float bsum[4][8];                                  // bias gradient: this lane's units, summed over its rows and all steps
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) bsum[g][e] = 0.0f;
    for (int v = tid; v < 16 * 256; v += 512) reinterpret_cast<u32x4 *>(dabuf)[v] = u32x4{0u, 0u, 0u, 0u};   // padding stays zero
    const bool active = hb < n_hb;                     // uniform over the wavefront
    const int col = lane & 31, rsub = (lane >> 5) * 4;
    const int irow = lane >> 2, igrp = (lane & 3) * 8; // item k of this lane: row irow + 16 k, units igrp..igrp + 7 of the block
    const int j8 = hb * 32 + igrp;
    const bool units8 = active && j8 < H;              // H % 8 == 0: a group of 8 is inside or outside
    const int kc8 = j8 >> 6, kk8 = j8 & 63;
#pragma unroll
    for (int k = 0; k < 4; ++k) dcl[k][tid] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    const int hbc = min(hb, n_hb - 1);
    // B fragments of this wavefront: chunk (nt, gate, c), k-step ks, unit block hbc % 4
    const u32x4 *UT = reinterpret_cast<const u32x4 *>(a.UTpk) + (int64_t)(hbc >> 2) * 4 * a.nkc * (B_CHUNK / 8) + (hbc & 3) * 64 + lane;
    const u32x4 *Ad = reinterpret_cast<const u32x4 *>(dabuf) + lane;
    float *tile = stage[hb];
    // U^T fragments of a half chunk (gate q % 4, half chunk q / 4): two per lane
    auto loadB = [&](u32x4 (&rb)[2], int q) {
        const int chunk = (q & 3) * a.nkc + (q >> 3), hf = (q >> 2) & 1;
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) rb[k2] = UT[(int64_t)chunk * (B_CHUNK / 8) + (hf * 2 + k2) * 256];
    };
    u32x4 rb0[2], rb1[2], rb2[2], rb3[2];
    loadB(rb0, 0); loadB(rb1, 1); loadB(rb2, 2); loadB(rb3, 3);
    u32x4 vct_next[2] = {};                            // c_{t-1} of step t is c_t of step t - 1
    __syncthreads();
    for (int t = a.T - 1; t >= 0; --t) {
        const bool first = t == a.T - 1;
        // this step's saved activations and the gradient from above do not depend on the recurrence: requested first
        u32x4 vi[2], vf[2], vg[2], vo[2], vct[2], vcp[2], vdh[2];
        bool ok[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int row = r0 + irow + 16 * k;
            ok[k] = units8 && row < a.B;
            if (ok[k]) {
                const T *gr = reinterpret_cast<const T *>(a.gates) + (int64_t)t * a.B * G + (int64_t)row * G + j8;
                const int64_t e = (int64_t)row * H + j8;
                vi[k] = *reinterpret_cast<const u32x4 *>(gr);
                vf[k] = *reinterpret_cast<const u32x4 *>(gr + H);
                vg[k] = *reinterpret_cast<const u32x4 *>(gr + 2 * H);
                vo[k] = *reinterpret_cast<const u32x4 *>(gr + 3 * H);
                vcp[k] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(a.cs) + (int64_t)t * a.B * H + e);
                vct[k] = first ? *reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(a.cs) + (int64_t)(t + 1) * a.B * H + e) : vct_next[k];
                vct_next[k] = vcp[k];
                vdh[k] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const T *>(a.dh_above) + (int64_t)t * a.B * H + e);
            }
        }
        v16f acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        if (active && !first) {
            // dh_rec = dA_{t+1} U for this block of units: four register sets of one half chunk each
            auto loadA = [&](u32x4 (&ra)[2], int q) {
                const int chunk = (q & 3) * a.nkc + (q >> 3), hf = (q >> 2) & 1;
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) ra[k2] = Ad[(chunk * 4 + hf * 2 + k2) * 64];
            };
            auto mm = [&](const u32x4 (&ra)[2], const u32x4 (&rb)[2]) {
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) acc = Lp<T>::mfma(ra[k2], rb[k2], acc);
            };
            u32x4 ra0[2], ra1[2], ra2[2], ra3[2];
            loadA(ra0, 0); loadA(ra1, 1); loadA(ra2, 2); loadA(ra3, 3);      // their weights are already in rb0 .. rb3
            int s = 0;
            for (; s + 8 <= nq; s += 4) {              // nq is a multiple of four; branch-free body
                mm(ra0, rb0); loadB(rb0, s + 4); loadA(ra0, s + 4);
                mm(ra1, rb1); loadB(rb1, s + 5); loadA(ra1, s + 5);
                mm(ra2, rb2); loadB(rb2, s + 6); loadA(ra2, s + 6);
                mm(ra3, rb3); loadB(rb3, s + 7); loadA(ra3, s + 7);
            }
            mm(ra0, rb0); loadB(rb0, 0);               // the next step's first weights travel during this step's epilogue
            mm(ra1, rb1); loadB(rb1, 1);
            mm(ra2, rb2); loadB(rb2, 2);
            mm(ra3, rb3); loadB(rb3, 3);
        }
        __syncthreads();                               // every wavefront has read dA_{t+1}: the buffer may take dA_t
        if (active) {
            // accumulator layout (lane = unit, 16 rows) -> item layout (lane = 8 units of rows irow, irow + 16)
#pragma unroll
            for (int r = 0; r < 16; ++r) tile[(rsub + (r >> 2) * 8 + (r & 3)) * SLD + col] = acc[r];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                if (!ok[k]) continue;
                const int rl = irow + 16 * k, row = r0 + rl;
                __attribute__((aligned(16))) float rec[8];
                *reinterpret_cast<v4f *>(rec) = *reinterpret_cast<const v4f *>(tile + rl * SLD + igrp);
                *reinterpret_cast<v4f *>(rec + 4) = *reinterpret_cast<const v4f *>(tile + rl * SLD + igrp + 4);
                __attribute__((aligned(16))) T ti[8], tf[8], tg[8], to[8], tct[8], tcp[8], tdh[8], o0[8], o1[8], o2[8], o3[8];
                *reinterpret_cast<u32x4 *>(ti) = vi[k]; *reinterpret_cast<u32x4 *>(tf) = vf[k]; *reinterpret_cast<u32x4 *>(tg) = vg[k];
                *reinterpret_cast<u32x4 *>(to) = vo[k]; *reinterpret_cast<u32x4 *>(tct) = vct[k]; *reinterpret_cast<u32x4 *>(tcp) = vcp[k];
                *reinterpret_cast<u32x4 *>(tdh) = vdh[k];
                __attribute__((aligned(16))) float dck[8];
                *reinterpret_cast<v4f *>(dck) = dcl[2 * k][tid];
                *reinterpret_cast<v4f *>(dck + 4) = dcl[2 * k + 1][tid];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float i = Lp<T>::to_f(ti[e]), f = Lp<T>::to_f(tf[e]), g = Lp<T>::to_f(tg[e]), o = Lp<T>::to_f(to[e]);
                    const float tc = tanhf_dev(Lp<T>::to_f(tct[e]));
                    const float dh = Lp<T>::to_f(tdh[e]) + rec[e];
                    const float d_o = dh * tc;
                    const float dcv = dck[e] + dh * o * (1.0f - tc * tc);
                    const float di = dcv * g, dg = dcv * i, df = dcv * Lp<T>::to_f(tcp[e]);
                    dck[e] = dcv * f;
                    const float a0 = di * i * (1.0f - i), a1 = df * f * (1.0f - f), a2 = dg * (1.0f - g * g), a3 = d_o * o * (1.0f - o);
                    o0[e] = Lp<T>::from_f(a0); o1[e] = Lp<T>::from_f(a1); o2[e] = Lp<T>::from_f(a2); o3[e] = Lp<T>::from_f(a3);
                    bsum[0][e] += a0; bsum[1][e] += a1; bsum[2][e] += a2; bsum[3][e] += a3;      // (before the rounding to 16 bits)
                }
                dcl[2 * k][tid] = *reinterpret_cast<const v4f *>(dck);
                dcl[2 * k + 1][tid] = *reinterpret_cast<const v4f *>(dck + 4);
                // the next step's operand: 8 units of a row and gate are one 16-byte slot of the fragment order
                u32x4 *slot = reinterpret_cast<u32x4 *>(dabuf) + (kc8 * 4 + (kk8 >> 4)) * 64 + ((kk8 >> 3) & 1) * 32 + rl;
                const int gs = a.nkc * 256;                // 16-byte slots per gate
                slot[0] = *reinterpret_cast<const u32x4 *>(o0);
                slot[gs] = *reinterpret_cast<const u32x4 *>(o1);
                slot[2 * gs] = *reinterpret_cast<const u32x4 *>(o2);
                slot[3 * gs] = *reinterpret_cast<const u32x4 *>(o3);
                if (a.dA) {
                    T *da = reinterpret_cast<T *>(a.dA) + (int64_t)t * a.B * G + (int64_t)row * G + j8;
                    *reinterpret_cast<u32x4 *>(da) = *reinterpret_cast<const u32x4 *>(o0);
                    *reinterpret_cast<u32x4 *>(da + H) = *reinterpret_cast<const u32x4 *>(o1);
                    *reinterpret_cast<u32x4 *>(da + 2 * H) = *reinterpret_cast<const u32x4 *>(o2);
                    *reinterpret_cast<u32x4 *>(da + 3 * H) = *reinterpret_cast<const u32x4 *>(o3);
                }
                if (a.dAblk) {
                    T *rowp = reinterpret_cast<T *>(a.dAblk) + (int64_t)t * a.slot_blk + (int64_t)mt * a.blk_ncb * 4096 + (mb * 32 + rl) * 64;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int cg = g * H + j8;
                        const T *src = g == 0 ? o0 : (g == 1 ? o1 : (g == 2 ? o2 : o3));
                        *reinterpret_cast<u32x4 *>(rowp + (int64_t)(cg >> 6) * 4096 + (cg & 63)) = *reinterpret_cast<const u32x4 *>(src);
                    }
                }
            }
        }
        __syncthreads();                               // dA_t of every unit block is in LDS
    }
    if (a.bias_partial) {
        // the sixteen lanes that share a group of 8 units (lane % 4) hold different rows: add them up
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v = bsum[g][e];
#pragma unroll
                for (int off = 4; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
                bsum[g][e] = v;
            }
        if (units8 && lane < 4) {
            float *dst = a.bias_partial + (int64_t)blockIdx.x * G + j8;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                *reinterpret_cast<v4f *>(dst + g * H) = v4f{bsum[g][0], bsum[g][1], bsum[g][2], bsum[g][3]};
                *reinterpret_cast<v4f *>(dst + g * H + 4) = v4f{bsum[g][4], bsum[g][5], bsum[g][6], bsum[g][7]};
            }
        }
    }
}

// ---------------------------------------------------------------- backward
struct BwdArgs {
    const void *dApk;      // packed dA_{t+1}: [n_mt][4][nkc][64][64]
    const void *UTpk;      // packed U^T: [n_nt][4][nkc][128][64]
    float *partials;       // fp32 [slices][B,H] out: one K-slice (gate) each, or the whole sum
    int B, H, n_mt, nkc;
    int slices;            // 4: the contraction over the 4H gate rows is split by gate over workgroups; 1: not split
};

// partial[q][b, j] = sum over the rows k of gate q of dA_next[b, k] * U[k, j]   (slices = 4)
// partial[0][b, j] = sum over all 4H rows                                        (slices = 1: enough tiles without the split)
template <typename T, bool WIDE>
__device__ __forceinline__ void backward_gemm_cell(const BwdArgs &a, int lin, int total, int rot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // gate-slice major: the workgroups of one XCD share one K slice, so that XCD's L2 pulls
    // only that quarter of dA over the fabric (all of it would be fetched by all eight otherwise)
    const int per_q = total / a.slices;
    const int q = lin / per_q, tile = lin - q * per_q;
    const int mt = tile % a.n_mt, nt = tile / a.n_mt;
    const int m0 = mt * TM, n0 = nt * TN;
    const int H = a.H;
    // the chunks of the four gates follow each other in both packed operands, so the unsplit
    // contraction is the same loop over four times as many chunks
    const int nch = a.slices == 1 ? 4 * a.nkc : a.nkc;
    const int cpw = (nch + 3) / 4;
    const int c0 = WIDE ? 0 : min(nch, wave * cpw), c1 = WIDE ? nch : min(nch, c0 + cpw);
    v16f acc[2][NBLK];
    zero_acc(acc);
    packed_mainloop<T>(reinterpret_cast<const uint16_t *>(a.dApk) + ((int64_t)mt * 4 + q) * a.nkc * A_CHUNK,
                       reinterpret_cast<const uint16_t *>(a.UTpk) + ((int64_t)nt * 4 + q) * a.nkc * B_CHUNK, c0, c1, rot, lane, acc);
    float *part = a.partials + (int64_t)q * a.B * H;
    auto store_group = [&](int mb, int rh, const float (&sum)[8][NBLK]) {
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int r = rh + rr;
            const int row = m0 + mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row >= a.B) continue;
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb) {
                const int j = n0 + nb * 32 + (lane & 31);
                if (j < H) part[(int64_t)row * H + j] = sum[rr][nb];
            }
        }
    };
    if constexpr (WIDE) {
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int mb = grp >> 1, rh = (grp & 1) * 8;
            float sum[8][NBLK];
#pragma unroll
            for (int rr = 0; rr < 8; ++rr)
#pragma unroll
                for (int nb = 0; nb < NBLK; ++nb) sum[rr][nb] = acc[mb][nb][rh + rr];
            store_group(mb, rh, sum);
        }
    } else {
        __shared__ __attribute__((aligned(16))) float smem[4 * RED_FLOATS];
        float sum[8][NBLK];
        reduce_waves(smem, wave, lane, acc, sum);
        store_group(wave >> 1, (wave & 1) * 8, sum);
    }
}

template <typename T, bool WIDE>
__global__ __launch_bounds__(256) void lstm_step_backward_gemm_kernel(BwdArgs a) {
    backward_gemm_cell<T, WIDE>(a, xcd_swizzle(blockIdx.x, gridDim.x), (int)gridDim.x, (int)blockIdx.x);
}

// Several products in one launch (the backward anti-diagonal: dA_t U of every ready layer, and
// dA_t W for the layer below it).
constexpr int WAVE_MAX_GEMMS = 16;
struct WaveBwdGemmArgs {
    const void *dApk[WAVE_MAX_GEMMS];
    const void *Bpk[WAVE_MAX_GEMMS];
    float *partials[WAVE_MAX_GEMMS];
    int B, H, n_mt, nkc, wgs_per_cell;
};
template <typename T>
__global__ __launch_bounds__(256) void lstm_wave_backward_gemm_kernel(WaveBwdGemmArgs w) {
    const int c = blockIdx.x / w.wgs_per_cell;
    BwdArgs a;
    a.dApk = w.dApk[c]; a.UTpk = w.Bpk[c]; a.partials = w.partials[c];
    a.B = w.B; a.H = w.H; a.n_mt = w.n_mt; a.nkc = w.nkc; a.slices = 4;
    backward_gemm_cell<T, false>(a, (int)blockIdx.x - c * w.wgs_per_cell, w.wgs_per_cell, (int)blockIdx.x);
}

// BPTT through the gates of one step; sums the four recurrent partials, writes
// dA row-major (for the whole-sequence GEMMs) and packed (A operand of the next
// recurrent GEMM).  VEC: H % 8 == 0 and 16-byte aligned tensors; one thread
// owns 8 consecutive hidden units of one batch row (16-byte loads and stores,
// and its 8 packed outputs are one 16-byte fragment slot).
// The gradient arriving from above is dh_above (16-bit, row-major: the head or a whole-sequence
// data-gradient GEMM) and/or above4 (four fp32 K-slice partials of the per-step product
// dA_t W of the layer above, used when the backward pass runs along anti-diagonals).
template <typename T, int W>
__device__ __forceinline__ void gates_backward_cell(const T *dh_above, const float *above4, const float *partials, const T *gates,
                                                    const T *c_t, const T *c_prev, float *dc_state, T *dA, T *dApk, T *dAblk,
                                                    int blk_ncb, int B, int H, int nkc, int first, int64_t thread0,
                                                    int64_t nthreads, int n_part = 4) {
    constexpr bool VEC = W > 1;
    typedef unsigned int lpvec __attribute__((ext_vector_type(W > 1 ? W / 2 : 1)));   // W 16-bit values
    const int64_t n = (int64_t)B * H;
    const int G = 4 * H;
    const int64_t gs = (int64_t)nkc * A_CHUNK;
    // Which 8 units a thread takes.  Plain: consecutive threads walk along a row.  With whole 8 x 64 patches
    // (B % 8 == 0, H % 64 == 0) a wavefront takes 8 rows x 64 units instead, lane = row + 8 * group of 8 units:
    // its loads and row-major stores are still whole 128-byte lines (8 lanes side by side in a row), and so are its
    // stores into the packed copy, where a line holds one group of 8 units of 8 consecutive rows (with the plain
    // order those eight 16-byte pieces come from eight workgroups on as many XCDs and reach memory one by one).
    const bool patches = VEC && W == 8 && B % 8 == 0 && H % 64 == 0;
    for (int64_t it = thread0; it * W < n; it += nthreads) {
        int64_t e0 = it * W;
        if (patches) {
            const int64_t patch = it >> 6;
            const int lane = (int)(it & 63), per_row = H >> 6;
            e0 = ((patch / per_row) * 8 + (lane & 7)) * (int64_t)H + (patch % per_row) * 64 + (lane >> 3) * 8;
        }
        const int b = (int)(e0 / H), j0 = (int)(e0 % H);
        __attribute__((aligned(16))) T vi[W], vf[W], vg[W], vo[W], vct[W], vcp[W], vdh[W];
        __attribute__((aligned(16))) float p0[W], p1[W], p2[W], p3[W], dcs[W];
        const T *gr = gates + (int64_t)b * G + j0;
        if constexpr (VEC) {
            *reinterpret_cast<lpvec *>(vi) = *reinterpret_cast<const lpvec *>(gr);
            *reinterpret_cast<lpvec *>(vf) = *reinterpret_cast<const lpvec *>(gr + H);
            *reinterpret_cast<lpvec *>(vg) = *reinterpret_cast<const lpvec *>(gr + 2 * H);
            *reinterpret_cast<lpvec *>(vo) = *reinterpret_cast<const lpvec *>(gr + 3 * H);
            *reinterpret_cast<lpvec *>(vct) = *reinterpret_cast<const lpvec *>(c_t + e0);
            *reinterpret_cast<lpvec *>(vcp) = *reinterpret_cast<const lpvec *>(c_prev + e0);
            if (dh_above) *reinterpret_cast<lpvec *>(vdh) = *reinterpret_cast<const lpvec *>(dh_above + e0);
            if (!first) {
#pragma unroll
                for (int h = 0; h < W / 4; ++h) {
                    *reinterpret_cast<u32x4 *>(p0 + 4 * h) = *reinterpret_cast<const u32x4 *>(partials + e0 + 4 * h);
                    if (n_part >= 2) *reinterpret_cast<u32x4 *>(p1 + 4 * h) = *reinterpret_cast<const u32x4 *>(partials + n + e0 + 4 * h);
                    if (n_part == 4) {
                        *reinterpret_cast<u32x4 *>(p2 + 4 * h) = *reinterpret_cast<const u32x4 *>(partials + 2 * n + e0 + 4 * h);
                        *reinterpret_cast<u32x4 *>(p3 + 4 * h) = *reinterpret_cast<const u32x4 *>(partials + 3 * n + e0 + 4 * h);
                    }
                    *reinterpret_cast<u32x4 *>(dcs + 4 * h) = *reinterpret_cast<const u32x4 *>(dc_state + e0 + 4 * h);
                }
            }
        } else {
            vi[0] = gr[0]; vf[0] = gr[H]; vg[0] = gr[2 * H]; vo[0] = gr[3 * H];
            vct[0] = c_t[e0]; vcp[0] = c_prev[e0];
            if (dh_above) vdh[0] = dh_above[e0];
            if (!first) {
                p0[0] = partials[e0];
                if (n_part >= 2) p1[0] = partials[n + e0];
                if (n_part == 4) { p2[0] = partials[2 * n + e0]; p3[0] = partials[3 * n + e0]; }
                dcs[0] = dc_state[e0];
            }
        }
        __attribute__((aligned(16))) T o0[W], o1[W], o2[W], o3[W];
        __attribute__((aligned(16))) float dcn[W];
#pragma unroll
        for (int k = 0; k < W; ++k) {
            const float i = Lp<T>::to_f(vi[k]), f = Lp<T>::to_f(vf[k]), g = Lp<T>::to_f(vg[k]), o = Lp<T>::to_f(vo[k]);
            const float tc = tanhf_dev(Lp<T>::to_f(vct[k]));
            float dh = dh_above ? Lp<T>::to_f(vdh[k]) : 0.0f;
            if (above4) dh += (above4[e0 + k] + above4[n + e0 + k]) + (above4[2 * n + e0 + k] + above4[3 * n + e0 + k]);
            float dcr = 0.0f;
            if (!first) {
                dh += n_part == 4 ? (p0[k] + p1[k]) + (p2[k] + p3[k]) : (n_part == 2 ? p0[k] + p1[k] : p0[k]);
                dcr = dcs[k];
            }
            const float d_o = dh * tc;
            const float dc = dcr + dh * o * (1.0f - tc * tc);
            const float di = dc * g, dg = dc * i, df = dc * Lp<T>::to_f(vcp[k]);
            dcn[k] = dc * f;
            o0[k] = Lp<T>::from_f(di * i * (1.0f - i));
            o1[k] = Lp<T>::from_f(df * f * (1.0f - f));
            o2[k] = Lp<T>::from_f(dg * (1.0f - g * g));
            o3[k] = Lp<T>::from_f(d_o * o * (1.0f - o));
        }
        T *da = dA + (int64_t)b * G + j0;
        // packed: [b / 64][gate][j / 64] chunk, fragment order inside; 8 aligned units are one slot
        T *pk = dApk + (((int64_t)(b >> 6) * 4) * nkc + (j0 >> 6)) * A_CHUNK + frag_offset(b & 63, j0 & 63, 2);
        if constexpr (VEC) {
            if (dA) {                                  // row-major copy only where somebody reads it
                *reinterpret_cast<lpvec *>(da) = *reinterpret_cast<const lpvec *>(o0);
                *reinterpret_cast<lpvec *>(da + H) = *reinterpret_cast<const lpvec *>(o1);
                *reinterpret_cast<lpvec *>(da + 2 * H) = *reinterpret_cast<const lpvec *>(o2);
                *reinterpret_cast<lpvec *>(da + 3 * H) = *reinterpret_cast<const lpvec *>(o3);
            }
            *reinterpret_cast<lpvec *>(pk) = *reinterpret_cast<const lpvec *>(o0);
            *reinterpret_cast<lpvec *>(pk + gs) = *reinterpret_cast<const lpvec *>(o1);
            *reinterpret_cast<lpvec *>(pk + 2 * gs) = *reinterpret_cast<const lpvec *>(o2);
            *reinterpret_cast<lpvec *>(pk + 3 * gs) = *reinterpret_cast<const lpvec *>(o3);
#pragma unroll
            for (int h = 0; h < W / 4; ++h) *reinterpret_cast<u32x4 *>(dc_state + e0 + 4 * h) = *reinterpret_cast<const u32x4 *>(dcn + 4 * h);
        } else {
            if (dA) { da[0] = o0[0]; da[H] = o1[0]; da[2 * H] = o2[0]; da[3 * H] = o3[0]; }
            pk[0] = o0[0]; pk[gs] = o1[0]; pk[2 * gs] = o2[0]; pk[3 * gs] = o3[0];
            dc_state[e0] = dcn[0];
        }
        if (dAblk) {
            // 64x64-blocked copy for the whole-sequence GEMMs: row b of this time slot, column gate*H + j
            T *rowp = dAblk + (int64_t)(b >> 6) * blk_ncb * 4096 + (b & 63) * 64;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = g * H + j0;
                T *d = rowp + (int64_t)(col >> 6) * 4096 + (col & 63);
                const T *src = g == 0 ? o0 : (g == 1 ? o1 : (g == 2 ? o2 : o3));
                if constexpr (VEC) *reinterpret_cast<lpvec *>(d) = *reinterpret_cast<const lpvec *>(src);
                else d[0] = src[0];
            }
        }
    }
}

template <typename T, int W>
__global__ __launch_bounds__(256) void gates_backward_packed_kernel(const T *dh_above, const float *partials, const T *gates,
                                                                    const T *c_t, const T *c_prev, float *dc_state, T *dA,
                                                                    T *dApk, T *dAblk, int blk_ncb, int B, int H, int nkc,
                                                                    int first, int n_part) {
    fetch_now(n_part);
    fetch_now(dh_above); fetch_now(partials); fetch_now(gates); fetch_now(c_t); fetch_now(c_prev); fetch_now(dc_state); fetch_now(dA);
    fetch_now(dApk); fetch_now(dAblk); fetch_now(blk_ncb); fetch_now(B); fetch_now(H); fetch_now(nkc); fetch_now(first);
    gates_backward_cell<T, W>(dh_above, nullptr, partials, gates, c_t, c_prev, dc_state, dA, dApk, dAblk, blk_ncb, B, H, nkc, first,
                                blockIdx.x * (int64_t)blockDim.x + threadIdx.x, (int64_t)gridDim.x * blockDim.x, n_part);
}

// The BPTT gate arithmetic of several independent (layer, time) cells in one launch.
constexpr int WAVE_MAX_GATES = 8;
struct WaveGateCell {
    const void *dh_above;     // lp [B,H] or null
    const float *above4;      // fp32 [4][B,H] or null
    const float *partials;    // fp32 [4][B,H]: dA_{t+1} U of this layer (unused when first)
    const void *gates, *c_t, *c_prev;
    float *dc_state;
    void *dA, *dApk, *dAblk;
    int first;
};
struct WaveGateArgs {
    WaveGateCell cell[WAVE_MAX_GATES];
    int blk_ncb, B, H, nkc, blocks_per_cell;
    int n_part;               // K-slice partials per cell: 4 (one per gate) or 2 (the wide-layer tile kernels)
};
template <typename T, int W>
__global__ __launch_bounds__(256) void wave_gates_backward_kernel(WaveGateArgs w) {
    const int ci = blockIdx.x / w.blocks_per_cell;
    const WaveGateCell &c = w.cell[ci];
    const int blk = (int)blockIdx.x - ci * w.blocks_per_cell;
    gates_backward_cell<T, W>((const T *)c.dh_above, c.above4, c.partials, (const T *)c.gates, (const T *)c.c_t, (const T *)c.c_prev,
                                c.dc_state, (T *)c.dA, (T *)c.dApk, (T *)c.dAblk, w.blk_ncb, w.B, w.H, w.nkc, c.first,
                                blk * (int64_t)blockDim.x + threadIdx.x, (int64_t)w.blocks_per_cell * blockDim.x, w.n_part);
}

// ---------------------------------------------------------------- narrow layers
// Narrow layers: a time step is a few small tiles, the launches of one sequence form a long
// dependent chain, and what a launch costs is its own latency: how many bytes each compute unit
// has to pull in (measured: the duration follows bytes per compute unit, at ~45 GB/s each), how
// many barriers and dependent memory round trips it has.  The two kernels below do a whole
// cell per launch on R x R tiles (R = 32 or 16, one workgroup each, so a cell spreads over many
// compute units), request the epilogue's operands before the products start, keep NS chunks
// of operands in flight, and use 16-byte accesses throughout (H % 8 == 0).
//   backward: the workgroup contracts over ALL 4H gate rows of dA_{t+1} U (and of dA_t W of
//             the layer above) itself, its four wavefronts splitting that range, so the gradient
//             reaching its units is complete inside the workgroup and the gate arithmetic follows
//             in the epilogue: one launch per BPTT cell instead of two.
//   forward : wavefront q computes gate q's pre-activations over the whole K range (nothing to
//             add up), the four gates meet through LDS.
// Operands are the packed ones of the other kernels; an R-row slice of a chunk is a few
// contiguous pieces of it.
constexpr int FUSED_MAX_CELLS = 16;         // cells per launch; the argument block comes in three sizes (NC = 2, 4, 16):
                                           // a launch pays for the size of its arguments (measured: 16 slots instead
                                           // of 8 cost a two-cell launch 7 %)
struct FusedBwdCell {
    const void *dApk_next, *UTpk, *dApk_above, *WTpk, *dh_above, *gates, *c_t, *c_prev;
    float *dc_state;
    void *dA, *dApk, *dAblk;
    int first;
};
template <int NC> struct FusedBwdArgs {
    FusedBwdCell cell[NC];
    int blk_ncb, B, H, nkc;
};
template <int NC> struct NarrowFwdArgs {
    FwdArgs cell[NC];
};

// The cell's argument block is copied into registers in one go: cell = blockIdx.z, tile = (blockIdx.x,
// blockIdx.y): no division by a loaded value first, every field fetched at the top (fetch_now).

// How an R x R tile maps onto the packed chunks ([k-step of 16][32-row block][lane][8]) and onto the
// MFMA that multiplies it: 32x32x16 (lane = 32 (k / 8) + row) or 16x16x32 (lane = 16 (k / 8) + row).
template <typename T, int R> struct NarrowGeo;
template <typename T> struct NarrowGeo<T, 32> {
    typedef v16f acc_t;
    static constexpr int NR = 16, STEPS = 4, A_STRIDE = 128, B_STRIDE = 256;   // strides in 16-byte units
    __device__ static int lane_a(int lane) { return lane; }
    __device__ static int lane_b(int lane) { return lane; }
    // 16-byte offset of rows r0.. of a 64-row A chunk / 128-row B chunk
    __device__ static int slice_a(int r0) { return ((r0 >> 5) & 1) * 64; }
    __device__ static int slice_b(int r0) { return ((r0 >> 5) & 3) * 64; }
    __device__ static int row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }
    __device__ static int col(int lane) { return lane & 31; }
    __device__ static acc_t mfma(const u32x4 &a, const u32x4 &b, acc_t c) { return Lp<T>::mfma(a, b, c); }
};
template <typename T> struct NarrowGeo<T, 16> {
    typedef v4f acc_t;
    static constexpr int NR = 4, STEPS = 2, A_STRIDE = 256, B_STRIDE = 512;
    // a 32-deep step spans two 16-deep k-steps of the chunk: lane / 32 picks the k-step, (lane / 16) % 2 its half
    __device__ static int lane_a(int lane) { return (lane >> 5) * 128 + ((lane >> 4) & 1) * 32 + (lane & 15); }
    __device__ static int lane_b(int lane) { return (lane >> 5) * 256 + ((lane >> 4) & 1) * 32 + (lane & 15); }
    __device__ static int slice_a(int r0) { return ((r0 >> 5) & 1) * 64 + ((r0 >> 4) & 1) * 16; }
    __device__ static int slice_b(int r0) { return ((r0 >> 5) & 3) * 64 + ((r0 >> 4) & 1) * 16; }
    __device__ static int row(int r, int lane) { return (lane >> 4) * 4 + r; }
    __device__ static int col(int lane) { return lane & 15; }
    __device__ static acc_t mfma(const u32x4 &a, const u32x4 &b, acc_t c) { return Lp<T>::mfma16(a, b, c); }
};

// acc += sum over the chunks k in [c0, c1) of the list [pair 1: n1 chunks][pair 2] of (R rows of the A
// chunk) x (R rows of the B chunk)^T; the pointers already address the slices and the lane.
template <typename T, int R, int NS>
__device__ __forceinline__ void narrow_mainloop(const u32x4 *A1, const u32x4 *B1, const u32x4 *A2, const u32x4 *B2, int n1, int c0,
                                                int c1, typename NarrowGeo<T, R>::acc_t &acc) {
    typedef NarrowGeo<T, R> Geo;
    constexpr int STEPS = Geo::STEPS, AV = A_CHUNK / 8, BV = B_CHUNK / 8;   // chunk sizes in 16-byte units
    if (c1 <= c0) return;
    auto load = [&](u32x4 (&ra)[STEPS], u32x4 (&rb)[STEPS], int k) {
        const u32x4 *a = k < n1 ? A1 + (int64_t)k * AV : A2 + (int64_t)(k - n1) * AV;
        const u32x4 *b = k < n1 ? B1 + (int64_t)k * BV : B2 + (int64_t)(k - n1) * BV;
#pragma unroll
        for (int i = 0; i < STEPS; ++i) ra[i] = a[Geo::A_STRIDE * i];
#pragma unroll
        for (int i = 0; i < STEPS; ++i) rb[i] = b[Geo::B_STRIDE * i];
    };
    auto mul = [&](const u32x4 (&ra)[STEPS], const u32x4 (&rb)[STEPS]) {
#pragma unroll
        for (int i = 0; i < STEPS; ++i) acc = Geo::mfma(ra[i], rb[i], acc);
    };
    u32x4 ra[NS][STEPS], rb[NS][STEPS];
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if (c0 + i < c1) load(ra[i], rb[i], c0 + i);
    int k = c0;
    for (; k + 2 * NS <= c1; k += NS) {        // branch-free body: every refill is in range
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            mul(ra[i], rb[i]);
            load(ra[i], rb[i], k + NS + i);
        }
    }
    // fewer than 2 NS chunks left; set i holds chunk k + i
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        if (k + i < c1) mul(ra[i], rb[i]);
        if (k + NS + i < c1) load(ra[i], rb[i], k + NS + i);
    }
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
        if (k + NS + i < c1) mul(ra[i], rb[i]);
}

// IW consecutive 16-bit values / floats as one access
template <int BYTES> struct VecOfBytes;
template <> struct VecOfBytes<16> { typedef u32x4 type; };
template <> struct VecOfBytes<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct VecOfBytes<4> { typedef unsigned int type; };
template <> struct VecOfBytes<2> { typedef unsigned short type; };
template <int BYTES, typename D, typename S>
__device__ __forceinline__ void copy_bytes(D *dst, const S *src) {
    if constexpr (BYTES == 32) {
        reinterpret_cast<u32x4 *>(dst)[0] = reinterpret_cast<const u32x4 *>(src)[0];
        reinterpret_cast<u32x4 *>(dst)[1] = reinterpret_cast<const u32x4 *>(src)[1];
    } else {
        typedef typename VecOfBytes<BYTES>::type V;
        *reinterpret_cast<V *>(dst) = *reinterpret_cast<const V *>(src);
    }
}

// One batch row x IW consecutive units of a BPTT cell (IW = 8, 4, 2 or 1; j0 a multiple of IW): operands
// requested early, finished once the gradient reaching h_t of those units (rec, from the products) is
// known.  These kernels are latency-bound, so IW is chosen to give every thread of the workgroup an item:
// what counts is the length of one thread's instruction stream, not the width of its accesses.
template <typename T, int IW> struct BackwardItem {
    __attribute__((aligned(16))) T vi[IW], vf[IW], vg[IW], vo[IW], vct[IW], vcp[IW], vdh[IW];
    __attribute__((aligned(16))) float dcs[IW];
    __device__ __forceinline__ void request(const FusedBwdCell &c, int b, int j0, int H) {
        const int64_t e0 = (int64_t)b * H + j0;
        const T *gr = reinterpret_cast<const T *>(c.gates) + (int64_t)b * 4 * H + j0;
        copy_bytes<2 * IW>(vi, gr);
        copy_bytes<2 * IW>(vf, gr + H);
        copy_bytes<2 * IW>(vg, gr + 2 * H);
        copy_bytes<2 * IW>(vo, gr + 3 * H);
        copy_bytes<2 * IW>(vct, reinterpret_cast<const T *>(c.c_t) + e0);
        copy_bytes<2 * IW>(vcp, reinterpret_cast<const T *>(c.c_prev) + e0);
        if (c.dh_above) copy_bytes<2 * IW>(vdh, reinterpret_cast<const T *>(c.dh_above) + e0);
        if (!c.first) copy_bytes<4 * IW>(dcs, c.dc_state + e0);
    }
    __device__ __forceinline__ void finish(const FusedBwdCell &c, const float (&rec)[IW], int b, int j0, int H, int nkc, int blk_ncb) {
        const int64_t e0 = (int64_t)b * H + j0;
        __attribute__((aligned(16))) T o0[IW], o1[IW], o2[IW], o3[IW];
        __attribute__((aligned(16))) float dcn[IW];
#pragma unroll
        for (int k = 0; k < IW; ++k) {
            const float i = Lp<T>::to_f(vi[k]), f = Lp<T>::to_f(vf[k]), g = Lp<T>::to_f(vg[k]), o = Lp<T>::to_f(vo[k]);
            const float tc = tanhf_dev(Lp<T>::to_f(vct[k]));
            const float dh = (c.dh_above ? Lp<T>::to_f(vdh[k]) : 0.0f) + rec[k];
            const float dcr = c.first ? 0.0f : dcs[k];
            const float d_o = dh * tc;
            const float dc = dcr + dh * o * (1.0f - tc * tc);
            const float di = dc * g, dg = dc * i, df = dc * Lp<T>::to_f(vcp[k]);
            dcn[k] = dc * f;
            o0[k] = Lp<T>::from_f(di * i * (1.0f - i));
            o1[k] = Lp<T>::from_f(df * f * (1.0f - f));
            o2[k] = Lp<T>::from_f(dg * (1.0f - g * g));
            o3[k] = Lp<T>::from_f(d_o * o * (1.0f - o));
        }
        // packed: [b / 64][gate][j / 64] chunk, fragment order inside; 8 aligned units are one 16-byte slot
        const int64_t gs = (int64_t)nkc * A_CHUNK;
        T *pk = reinterpret_cast<T *>(c.dApk) + (((int64_t)(b >> 6) * 4) * nkc + (j0 >> 6)) * A_CHUNK + frag_offset(b & 63, j0 & 63, 2);
        copy_bytes<2 * IW>(pk, o0);
        copy_bytes<2 * IW>(pk + gs, o1);
        copy_bytes<2 * IW>(pk + 2 * gs, o2);
        copy_bytes<2 * IW>(pk + 3 * gs, o3);
        copy_bytes<4 * IW>(c.dc_state + e0, dcn);
        if (c.dA) {
            T *da = reinterpret_cast<T *>(c.dA) + (int64_t)b * 4 * H + j0;
            copy_bytes<2 * IW>(da, o0);
            copy_bytes<2 * IW>(da + H, o1);
            copy_bytes<2 * IW>(da + 2 * H, o2);
            copy_bytes<2 * IW>(da + 3 * H, o3);
        }
        if (c.dAblk) {
            T *rowp = reinterpret_cast<T *>(c.dAblk) + (int64_t)(b >> 6) * blk_ncb * 4096 + (b & 63) * 64;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = g * H + j0;
                const T *src = g == 0 ? o0 : (g == 1 ? o1 : (g == 2 ? o2 : o3));
                copy_bytes<2 * IW>(rowp + (int64_t)(col >> 6) * 4096 + (col & 63), src);
            }
        }
    }
};

template <typename T, int R, int NC>
__global__ __launch_bounds__(256) void lstm_fused_backward_kernel(FusedBwdArgs<NC> w) {
    typedef NarrowGeo<T, R> Geo;
    constexpr int IW = R * R / 256;                              // units per thread: every thread gets an item
    constexpr int UG = R / IW, LD = R + 4, NR = Geo::NR;         // items per row, LDS row pitch, accumulator registers
    const FusedBwdCell c = w.cell[blockIdx.z];                   // uniform: the cell's argument block
    fetch_now(c.dApk_next); fetch_now(c.UTpk); fetch_now(c.dApk_above); fetch_now(c.WTpk); fetch_now(c.dh_above); fetch_now(c.gates);
    fetch_now(c.c_t); fetch_now(c.c_prev); fetch_now(c.dc_state); fetch_now(c.dA); fetch_now(c.dApk); fetch_now(c.dAblk);
    fetch_now(c.first); fetch_now(w.B); fetch_now(w.H); fetch_now(w.nkc); fetch_now(w.blk_ncb);
    const int b0 = (int)blockIdx.x * R, u0 = (int)blockIdx.y * R;    // first batch row, first hidden unit
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int H = w.H;
    const int row = tid / UG, ug = tid % UG;
    const int b = b0 + row, j0 = u0 + ug * IW;
    const bool valid = b < w.B && j0 < H;
    BackwardItem<T, IW> item;
    if (valid) item.request(c, b, j0, H);
    // chunk list: [dA_{t+1} x U^T: 4 nkc chunks][dA_t(above) x W^T: 4 nkc chunks], either part may be absent
    const int per = 4 * w.nkc;
    const int n1 = c.dApk_next ? per : 0, nch = n1 + (c.dApk_above ? per : 0);
    const int cpw = (nch + 3) / 4;
    const int c0 = min(nch, wave * cpw), c1 = min(nch, c0 + cpw);
    const int64_t a_off = (int64_t)(b0 >> 6) * per * (A_CHUNK / 8) + Geo::slice_a(b0) + Geo::lane_a(lane);
    const int64_t b_off = (int64_t)(u0 >> 7) * per * (B_CHUNK / 8) + Geo::slice_b(u0) + Geo::lane_b(lane);
    typename Geo::acc_t acc;
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.0f;
    narrow_mainloop<T, R, 4>(reinterpret_cast<const u32x4 *>(c.dApk_next) + a_off, reinterpret_cast<const u32x4 *>(c.UTpk) + b_off,
                             reinterpret_cast<const u32x4 *>(c.dApk_above) + a_off, reinterpret_cast<const u32x4 *>(c.WTpk) + b_off, n1,
                             c0, c1, acc);
    // sum the four wavefronts' accumulators and lay the tile out row by row
    __shared__ __attribute__((aligned(16))) float red[4 * NR * 64];
    __shared__ __attribute__((aligned(16))) float sums[R * LD];
#pragma unroll
    for (int r = 0; r < NR; ++r) red[(wave * NR + r) * 64 + lane] = acc[r];
    __syncthreads();
    for (int e = tid; e < NR * 64; e += 256) {
        const float v = (red[e] + red[NR * 64 + e]) + (red[2 * NR * 64 + e] + red[3 * NR * 64 + e]);
        sums[Geo::row(e >> 6, e & 63) * LD + Geo::col(e & 63)] = v;
    }
    __syncthreads();
    if (!valid) return;
    __attribute__((aligned(16))) float rec[IW];
    copy_bytes<4 * IW>(rec, sums + row * LD + ug * IW);
    item.finish(c, rec, b, j0, H, w.nkc, w.blk_ncb);
}

// One batch row x IW consecutive units of a forward cell.
template <typename T, int IW> struct ForwardItem {
    __attribute__((aligned(16))) T vax[4][IW];
    __attribute__((aligned(16))) float cprev[IW];
    __device__ __forceinline__ void request(const FwdArgs &a, int b, int j0) {
        const int H = a.H;
        // input projection (bias included) of this step, or just the bias when the cell projects its own input
        const T *ax = a.Ax ? reinterpret_cast<const T *>(a.Ax) + (int64_t)b * 4 * H + j0 : reinterpret_cast<const T *>(a.bias) + j0;
#pragma unroll
        for (int g = 0; g < 4; ++g) copy_bytes<2 * IW>(vax[g], ax + g * H);
        copy_bytes<4 * IW>(cprev, a.c_state + (int64_t)b * H + j0);
    }
    __device__ __forceinline__ void finish(const FwdArgs &a, const float (&pz)[4][IW], int b, int j0) {
        const int H = a.H;
        const int64_t e0 = (int64_t)b * H + j0;
        __attribute__((aligned(16))) T oi[IW], of[IW], og[IW], oo[IW], oc[IW], oh[IW];
        __attribute__((aligned(16))) float cn[IW];
#pragma unroll
        for (int k = 0; k < IW; ++k) {
            const float gi = sigmoidf_dev(pz[0][k] + Lp<T>::to_f(vax[0][k]));
            const float gf = sigmoidf_dev(pz[1][k] + Lp<T>::to_f(vax[1][k]));
            const float gg = tanhf_dev(pz[2][k] + Lp<T>::to_f(vax[2][k]));
            const float go = sigmoidf_dev(pz[3][k] + Lp<T>::to_f(vax[3][k]));
            const float cc = gf * cprev[k] + gi * gg;
            cn[k] = cc;
            oi[k] = Lp<T>::from_f(gi); of[k] = Lp<T>::from_f(gf); og[k] = Lp<T>::from_f(gg); oo[k] = Lp<T>::from_f(go);
            oc[k] = Lp<T>::from_f(cc);
            oh[k] = Lp<T>::from_f(go * tanhf_dev(cc));
        }
        copy_bytes<4 * IW>(a.c_state + e0, cn);
        T *gr = reinterpret_cast<T *>(a.gates) + (int64_t)b * 4 * H + j0;
        copy_bytes<2 * IW>(gr, oi);
        copy_bytes<2 * IW>(gr + H, of);
        copy_bytes<2 * IW>(gr + 2 * H, og);
        copy_bytes<2 * IW>(gr + 3 * H, oo);
        copy_bytes<2 * IW>(reinterpret_cast<T *>(a.c_out) + e0, oc);
        copy_bytes<2 * IW>(reinterpret_cast<T *>(a.h_out) + e0, oh);
        copy_bytes<2 * IW>(reinterpret_cast<T *>(a.hpk_next) + ((int64_t)(b >> 6) * a.nkc + (j0 >> 6)) * A_CHUNK + frag_offset(b & 63, j0 & 63, 2), oh);
        if (a.h_blk)
            copy_bytes<2 * IW>(reinterpret_cast<T *>(a.h_blk) + ((int64_t)(b >> 6) * a.blk_ncb + (j0 >> 6)) * 4096 + (b & 63) * 64 + (j0 & 63), oh);
    }
};

template <typename T, int R, int NC>
__global__ __launch_bounds__(256) void lstm_narrow_forward_kernel(NarrowFwdArgs<NC> w) {
    typedef NarrowGeo<T, R> Geo;
    constexpr int IW = R * R / 256;                              // units per thread: every thread gets an item
    constexpr int UG = R / IW, LD = R + 4, NR = Geo::NR;
    const FwdArgs a = w.cell[blockIdx.z];
    fetch_now(a.hpk_prev); fetch_now(a.Upk); fetch_now(a.Ax); fetch_now(a.xpk); fetch_now(a.Wpk); fetch_now(a.bias);
    fetch_now(a.c_state); fetch_now(a.gates); fetch_now(a.c_out); fetch_now(a.h_out); fetch_now(a.hpk_next); fetch_now(a.h_blk);
    fetch_now(a.blk_ncb); fetch_now(a.B); fetch_now(a.H); fetch_now(a.nkc);
    const int b0 = (int)blockIdx.x * R, u0 = (int)blockIdx.y * R;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = tid / UG, ug = tid % UG;
    const int b = b0 + row, j0 = u0 + ug * IW;
    const bool valid = b < a.B && j0 < a.H;
    ForwardItem<T, IW> item;
    if (valid) item.request(a, b, j0);
    const int nch = a.Ax ? a.nkc : a.nkc + a.nkc2;       // nkc2 = nkc here: the input of these cells is H wide
    // rows of U (and W): hidden block u0 / 32, inside it gate `wave`'s 32 rows, of those the tile's R
    const int64_t a_off = (int64_t)(b0 >> 6) * a.nkc * (A_CHUNK / 8) + Geo::slice_a(b0) + Geo::lane_a(lane);
    const int64_t b_off = (int64_t)(u0 >> 5) * a.nkc * (B_CHUNK / 8) + Geo::slice_b(wave * 32 + (u0 & 31)) + Geo::lane_b(lane);
    typename Geo::acc_t acc;
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.0f;
    narrow_mainloop<T, R, 4>(reinterpret_cast<const u32x4 *>(a.hpk_prev) + a_off, reinterpret_cast<const u32x4 *>(a.Upk) + b_off,
                             reinterpret_cast<const u32x4 *>(a.xpk) + a_off, reinterpret_cast<const u32x4 *>(a.Wpk) + b_off, a.nkc, 0,
                             nch, acc);
    __shared__ __attribute__((aligned(16))) float pre[4 * R * LD];     // [gate][row][unit]
#pragma unroll
    for (int r = 0; r < NR; ++r) pre[(wave * R + Geo::row(r, lane)) * LD + Geo::col(lane)] = acc[r];
    __syncthreads();
    if (!valid) return;
    __attribute__((aligned(16))) float pz[4][IW];
#pragma unroll
    for (int g = 0; g < 4; ++g) copy_bytes<4 * IW>(pz[g], pre + (g * R + row) * LD + ug * IW);
    item.finish(a, pz, b, j0);
}

// ---------------------------------------------------------------- fused backward step, large batches
// With thousands of rows per step the 64x128 tiles alone fill the chip, the contraction over the 4H gate rows
// is not split over workgroups (backward_slices), and the workgroup that owns a tile has the complete
// gradient of its 64 rows x 128 units: the gate arithmetic follows in its epilogue instead of in a second
// kernel, and the fp32 partial sums never go to memory.  Main loop and reduction are those of
// lstm_step_backward_gemm_kernel, the epilogue is BackwardItem's (four items of 8 units per thread).
struct FusedStepArgs {
    FusedBwdCell c;        // dApk_above / WTpk unused (the gradient from above arrives in dh_above)
    int blk_ncb, B, H, n_mt, nkc;
};
template <typename T>
__global__ __launch_bounds__(256) void lstm_step_backward_fused_kernel(FusedStepArgs a) {
    constexpr int LD = TN + 4;
    __shared__ __attribute__((aligned(16))) float smem[4 * RED_FLOATS];
    const FusedBwdCell c = a.c;
    const int lin = xcd_swizzle(blockIdx.x, gridDim.x);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = lin % a.n_mt, nt = lin / a.n_mt;
    const int m0 = mt * TM, n0 = nt * TN;
    const int H = a.H;
    const int nch = c.dApk_next ? 4 * a.nkc : 0;
    const int cpw = (nch + 3) / 4;
    const int c0 = min(nch, wave * cpw), c1 = min(nch, c0 + cpw);
    v16f acc[2][NBLK];
    zero_acc(acc);
    packed_mainloop<T>(reinterpret_cast<const uint16_t *>(c.dApk_next) + (int64_t)mt * 4 * a.nkc * A_CHUNK,
                       reinterpret_cast<const uint16_t *>(c.UTpk) + (int64_t)nt * 4 * a.nkc * B_CHUNK, c0, c1, (int)blockIdx.x, lane, acc);
    // the epilogue's operands: item i of this thread is batch row (i * 256 + tid) / 16 of the tile, units 8 ((i * 256 + tid) % 16) ..
    BackwardItem<T, 8> item[4];
    bool valid[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = i * 256 + tid, b = m0 + (idx >> 4), j0 = n0 + (idx & 15) * 8;
        valid[i] = b < a.B && j0 < H;
        if (valid[i]) item[i].request(c, b, j0, H);
    }
    float sum[8][NBLK];
    reduce_waves(smem, wave, lane, acc, sum);
    __syncthreads();                                   // every wavefront has read the partial sums
    {
        const int mb = wave >> 1, rh = (wave & 1) * 8;
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const int r = rh + rr, trow = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
#pragma unroll
            for (int nb = 0; nb < NBLK; ++nb) smem[trow * LD + nb * 32 + (lane & 31)] = sum[rr][nb];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (!valid[i]) continue;
        const int idx = i * 256 + tid, row = idx >> 4, ug = idx & 15;
        __attribute__((aligned(16))) float rec[8];
        copy_bytes<32>(rec, smem + row * LD + ug * 8);
        item[i].finish(c, rec, m0 + row, n0 + ug * 8, H, a.nkc, a.blk_ncb);
    }
}

// ---------------------------------------------------------------- packing
// chunk (hb, kc) of Upk, row g*32 + r, column kk = U[g*H + hb*32 + r][kc*64 + kk], zero outside;
// U is [4H, K] (K = H for the recurrent matrix, the layer's input width for W), nkc = ceil(K / 64)
template <typename T>
__device__ __forceinline__ void pack_u_forward_block(const T *U, T *Upk, int H, int nkc, int kc, int hb, int K) {
    T *dst = Upk + ((int64_t)hb * nkc + kc) * B_CHUNK;
    if (hb * 32 + 32 <= H && kc * 64 + 64 <= K && K % 8 == 0 && ((uintptr_t)U | (uintptr_t)Upk) % 16 == 0) {
        // whole chunk inside the matrix: 16-byte slots (8 consecutive k of one row), written in slot order
        for (int s = threadIdx.x; s < B_CHUNK / 8; s += 256) {
            const int r = s & 31, half = (s >> 5) & 1, g = (s >> 6) & (NBLK - 1), ks = s >> 8;
            const T *src = U + ((int64_t)g * H + hb * 32 + r) * K + kc * 64 + ks * 16 + half * 8;
            *reinterpret_cast<u32x4 *>(dst + s * 8) = *reinterpret_cast<const u32x4 *>(src);
        }
        return;
    }
    for (int v = threadIdx.x; v < B_CHUNK; v += 256) {
        const int row = v >> 6, kk = v & 63;
        const int g = row >> 5, r = row & 31;
        const int unit = hb * 32 + r, k = kc * 64 + kk;
        dst[frag_offset(row, kk, NBLK)] = (unit < H && k < K) ? U[((int64_t)g * H + unit) * K + k] : Lp<T>::from_f(0.0f);
    }
}
// chunk (nt, q, kc) of UTpk, row r, column kk = U[q*H + kc*64 + kk][nt*128 + r], zero outside
template <typename T>
__device__ __forceinline__ void pack_u_backward_block(const T *U, T *UTpk, int H, int nkc, int kc, int q, int nt, T (*tile)[TN + 2]) {
    // read U rows (k) x columns (units) coalesced along units, write transposed
    T *dst = UTpk + (((int64_t)nt * 4 + q) * nkc + kc) * B_CHUNK;
    if (kc * 64 + 64 <= H && nt * TN + TN <= H && H % 8 == 0 && ((uintptr_t)U | (uintptr_t)UTpk) % 16 == 0) {
        // whole chunk inside the matrix: 16 bytes (8 units of one k) per load, 16-byte slots (8 k of one unit) per store
        for (int v = threadIdx.x; v < 64 * TN / 8; v += 256) {
            const int kk = v / (TN / 8), r8 = (v % (TN / 8)) * 8;
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(U + ((int64_t)q * H + kc * 64 + kk) * H + nt * TN + r8);
            unsigned *t32 = reinterpret_cast<unsigned *>(&tile[kk][r8]);       // rows of the tile are 4-byte aligned
            t32[0] = raw[0]; t32[1] = raw[1]; t32[2] = raw[2]; t32[3] = raw[3];
        }
        __syncthreads();
        for (int s = threadIdx.x; s < B_CHUNK / 8; s += 256) {
            const int r = s & 31, half = (s >> 5) & 1, blk = (s >> 6) & (NBLK - 1), ks = s >> 8;
            const int row = blk * 32 + r, kk0 = ks * 16 + half * 8;
            __attribute__((aligned(16))) T o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = tile[kk0 + j][row];
            *reinterpret_cast<u32x4 *>(dst + s * 8) = *reinterpret_cast<const u32x4 *>(o);
        }
        return;
    }
    for (int v = threadIdx.x; v < 64 * TN; v += 256) {
        const int kk = v / TN, r = v % TN;
        const int k = kc * 64 + kk, unit = nt * TN + r;
        tile[kk][r] = (k < H && unit < H) ? U[((int64_t)q * H + k) * H + unit] : Lp<T>::from_f(0.0f);
    }
    __syncthreads();
    for (int v = threadIdx.x; v < B_CHUNK; v += 256) dst[frag_offset(v >> 6, v & 63, NBLK)] = tile[v & 63][v >> 6];
}
// chunk (mt, kc) of hpk, row, column kk = h[mt*64 + row][kc*64 + kk] (null h = 0), zero outside; h is [B, H]
template <typename T>
__device__ __forceinline__ void pack_rows_block(const T *h, T *hpk, int B, int H, int nkc, int kc, int mt) {
    T *dst = hpk + ((int64_t)mt * nkc + kc) * A_CHUNK;
    if (h && mt * 64 + 64 <= B && kc * 64 + 64 <= H && H % 8 == 0 && ((uintptr_t)h | (uintptr_t)hpk) % 16 == 0) {
        // whole chunk inside the matrix: 16-byte slots (8 consecutive k of one row), written in slot order
        for (int s = threadIdx.x; s < A_CHUNK / 8; s += 256) {
            const int r = s & 31, half = (s >> 5) & 1, blk = (s >> 6) & 1, ks = s >> 7;
            const T *src = h + (int64_t)(mt * 64 + blk * 32 + r) * H + kc * 64 + ks * 16 + half * 8;
            *reinterpret_cast<u32x4 *>(dst + s * 8) = *reinterpret_cast<const u32x4 *>(src);
        }
        return;
    }
    for (int v = threadIdx.x; v < A_CHUNK; v += 256) {
        const int row = mt * 64 + (v >> 6), k = kc * 64 + (v & 63);
        dst[frag_offset(v >> 6, v & 63, 2)] = (h && row < B && k < H) ? h[(int64_t)row * H + k] : Lp<T>::from_f(0.0f);
    }
}
// a whole sequence [T, B, K] packed step by step: blockIdx.z = time step
template <typename T>
__global__ __launch_bounds__(256) void pack_rows_seq_kernel(const T *x, T *xpk, int B, int K, int nkc, int64_t dst_stride) {
    pack_rows_block<T>(x + (int64_t)blockIdx.z * B * K, xpk + (int64_t)blockIdx.z * dst_stride, B, K, nkc, blockIdx.x, blockIdx.y);
}
template <typename T>
__global__ __launch_bounds__(256) void pack_u_forward_kernel(const T *U, T *Upk, int H, int nkc) {
    pack_u_forward_block<T>(U, Upk, H, nkc, blockIdx.x, blockIdx.y, H);
}
template <typename T>
__global__ __launch_bounds__(256) void pack_w_forward_kernel(const T *W, T *Wpk, int H, int K, int nkc) {
    pack_u_forward_block<T>(W, Wpk, H, nkc, blockIdx.x, blockIdx.y, K);
}
template <typename T>
__global__ __launch_bounds__(256) void pack_u_backward_kernel(const T *U, T *UTpk, int H, int nkc) {
    __shared__ T tile[64][TN + 2];
    pack_u_backward_block<T>(U, UTpk, H, nkc, blockIdx.x, blockIdx.y, blockIdx.z, tile);
}
template <typename T>
__global__ __launch_bounds__(256) void pack_rows_kernel(const T *h, T *hpk, int B, int H, int nkc) {
    pack_rows_block<T>(h, hpk, B, H, nkc, blockIdx.x, blockIdx.y);
}

// Several of the above (and plain fills) in one launch: blockIdx.y selects the job.  The set-up of a
// pass is a dozen small independent kernels, and on narrow layers every launch counts.
constexpr int SETUP_MAX_JOBS = 16;
struct SetupJobArg {
    const void *src;
    void *dst;
    int64_t n_words;
    int kind, ncb, cols;
};
struct SetupArgs {
    SetupJobArg job[SETUP_MAX_JOBS];
    int B, H, nkc, n_mt, n_hb, n_nt;
};
template <typename T>
__global__ __launch_bounds__(256) void setup_jobs_kernel(SetupArgs a) {
    __shared__ T tile[64][TN + 2];
    const SetupJobArg &j = a.job[blockIdx.y];
    const int x = blockIdx.x;
    switch (j.kind) {                                    // uniform over the workgroup
        case SETUP_PACK_U_FORWARD:
            if (x < a.nkc * a.n_hb) pack_u_forward_block<T>((const T *)j.src, (T *)j.dst, a.H, a.nkc, x % a.nkc, x / a.nkc, a.H);
            break;
        case SETUP_PACK_U_BACKWARD:
            if (x < a.nkc * 4 * a.n_nt)
                pack_u_backward_block<T>((const T *)j.src, (T *)j.dst, a.H, a.nkc, x % a.nkc, (x / a.nkc) & 3, x / (4 * a.nkc), tile);
            break;
        case SETUP_PACK_ROWS:
            if (x < a.nkc * a.n_mt) pack_rows_block<T>((const T *)j.src, (T *)j.dst, a.B, a.H, a.nkc, x % a.nkc, x / a.nkc);
            break;
        case SETUP_ZERO_PAD: {                           // padding columns of a 64x64-blocked 16-bit tensor
            const int c0 = j.cols & 63, npad = 64 - c0;
            const int64_t n = j.n_words * 64 * npad;     // row blocks x 64 rows x padding columns
            uint16_t *d = (uint16_t *)j.dst;
            if (c0 % 8 == 0) {                           // 16-byte pieces
                const int nv = npad / 8;
                for (int64_t i = (int64_t)x * 256 + threadIdx.x; i < n / 8; i += (int64_t)gridDim.x * 256) {
                    const int64_t r = i / nv;
                    const int c = c0 + (int)(i - r * nv) * 8;
                    *reinterpret_cast<u32x4 *>(d + ((r >> 6) * j.ncb + (j.ncb - 1)) * 4096 + (r & 63) * 64 + c) = u32x4{0u, 0u, 0u, 0u};
                }
                break;
            }
            for (int64_t i = (int64_t)x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
                const int64_t r = i / npad;              // row index over all row blocks
                const int c = c0 + (int)(i - r * npad);
                d[((r >> 6) * j.ncb + (j.ncb - 1)) * 4096 + (r & 63) * 64 + c] = 0;
            }
            break;
        }
        default: {                                       // SETUP_ZERO: n_words 32-bit words
            uint32_t *d = (uint32_t *)j.dst;
            for (int64_t i = (int64_t)x * 256 + threadIdx.x; i < j.n_words; i += (int64_t)gridDim.x * 256) d[i] = 0u;
        }
    }
}

}  // namespace

// ---------------------------------------------------------------- host side
RecurrentDims recurrent_dims(int B, int H) {
    RecurrentDims d;
    d.n_mt = (B + TM - 1) / TM;
    d.n_hb = (H + 31) / 32;
    d.n_nt = (H + TN - 1) / TN;
    d.nkc = (H + SK - 1) / SK;
    d.upk_elems = (size_t)d.n_hb * d.nkc * B_CHUNK;
    d.utpk_elems = (size_t)d.n_nt * 4 * d.nkc * B_CHUNK;
    d.hpk_elems = (size_t)d.n_mt * d.nkc * A_CHUNK;
    d.dapk_elems = (size_t)d.n_mt * 4 * d.nkc * A_CHUNK;
    d.partial_bytes = (size_t)4 * B * H * sizeof(float);
    return d;
}

// Few K chunks and many batch tiles: one-wavefront workgroups, one 64-row tile each over the
// whole K range, instead of a four-way K split with an LDS reduction.
// Narrow layers with a 16-byte-friendly width: the kernels that keep a whole cell in one launch.  Their
// backward form contracts over all 4H gate rows inside each workgroup, which stops paying above H = 768,
// and their small tiles re-read the operands too often once the batch is in the thousands (measured
// against the two-launch form: ahead or level for H <= 768 up to batch 4096 at H = 200..256, 1.6x behind
// at H = 2048, 12 % behind at H = 200 with 8192 rows).
// Shapes whose recurrences run as one launch per layer and direction (lstm_rows_*_kernel): at most eight blocks of
// 32 units, and enough 32-row groups to occupy the chip (measured against one launch per cell, 2 x 200 units,
// T = 128: 1024 rows 5.5 vs 3.4 ms per step, 2048 rows 6.4 vs 6.2, 4096 rows 8.4 vs 11.5, 6144 rows 10.7 vs 15.5).
// (Stacks of very narrow layers with at most 128 workgroups per cell keep the anti-diagonal schedule.)
static bool rows_shape(const RecurrentDims &d, int H) {
    return H % 8 == 0 && d.n_hb <= 8 && d.nkc <= 4 && d.n_mt >= 48 && d.n_mt * d.n_hb > 128;
}
static bool narrow_cells(const RecurrentDims &d, int H) { return H % 8 == 0 && H <= 768 && d.n_mt * d.n_hb <= 512 && !rows_shape(d, H); }
// Tile edge of the narrow-layer kernels: 16 while that keeps a launch (all its cells) within about 512
// workgroups: the smaller the tile, the fewer bytes each compute unit pulls in and the shorter the launch;
// with more cells per launch (deep stacks along the diagonals) the launch is bound by throughput and the
// 32x32 tile's lower operand traffic wins (measured, 200 units, batch 256: 2 layers 1.73 vs 1.90 ms per
// step with 16 vs 32, 12 layers 9.3 vs 7.8 ms, 29 layers 22.1 vs 18.7 ms).
static int narrow_tile(int B, int H, int n_cells) { return (int64_t)((B + 15) / 16) * ((H + 15) / 16) * n_cells <= 512 ? 16 : 32; }
// Slices of the backward contraction over the 4H gate rows: split by gate over four workgroups (four
// fp32 partial results that the gate kernel adds) unless the tiles alone fill the chip: then one
// workgroup contracts over all of it and 12 bytes per unit less are written and read back.
static int backward_slices(const RecurrentDims &d) { return d.n_mt * d.n_nt >= 256 ? 1 : 4; }
static bool recurrent_wide(const RecurrentDims &d) { return d.nkc <= 8 && d.n_mt >= 16; }   // H <= 512, B >= 961

#define LP_ONLY(dtype, T, ...)                                                       \
    if (dtype == LSTM_DTYPE_FP16) { using T = _Float16; __VA_ARGS__; }               \
    else if (dtype == LSTM_DTYPE_BF16) { using T = bf16_t; __VA_ARGS__; }            \
    else { set_error("recurrent kernels: dtype %d is not a 16-bit type", dtype); return LSTM_ERR_UNSUPPORTED; }

int pack_u_forward(int dtype, const void *U, void *Upk, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(1, H);
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_u_forward_kernel<T>, dim3(d.nkc, d.n_hb), dim3(256), 0, s, (const T *)U, (T *)Upk, H, d.nkc));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int pack_u_backward(int dtype, const void *U, void *UTpk, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(1, H);
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_u_backward_kernel<T>, dim3(d.nkc, 4, d.n_nt), dim3(256), 0, s, (const T *)U, (T *)UTpk, H, d.nkc));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int setup_jobs(int dtype, const SetupJob *jobs, int n_jobs, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    for (int first = 0; first < n_jobs; first += SETUP_MAX_JOBS) {
        const int n = n_jobs - first < SETUP_MAX_JOBS ? n_jobs - first : SETUP_MAX_JOBS;
        SetupArgs a;
        a.B = B; a.H = H; a.nkc = d.nkc; a.n_mt = d.n_mt; a.n_hb = d.n_hb; a.n_nt = d.n_nt;
        int64_t grid_x = 1;
        for (int i = 0; i < SETUP_MAX_JOBS; ++i) {
            const SetupJob &j = jobs[first + (i < n ? i : 0)];
            if (!j.dst || (j.kind < SETUP_PACK_ROWS && !j.src) || j.kind < 0 || j.kind > SETUP_ZERO_PAD ||
                (j.kind == SETUP_ZERO_PAD && (j.ncb < 1 || (j.cols & 63) == 0 || (j.cols + 63) / 64 != j.ncb))) {
                set_error("setup_jobs: bad job %d (kind %d)", first + i, j.kind);
                return LSTM_ERR_INVALID;
            }
            a.job[i].src = j.src; a.job[i].dst = j.dst; a.job[i].n_words = j.n_words; a.job[i].kind = j.kind;
            a.job[i].ncb = j.ncb; a.job[i].cols = j.cols;
            int64_t need = 1;
            switch (j.kind) {
                case SETUP_PACK_U_FORWARD: need = (int64_t)d.nkc * d.n_hb; break;
                case SETUP_PACK_U_BACKWARD: need = (int64_t)d.nkc * 4 * d.n_nt; break;
                case SETUP_PACK_ROWS: need = (int64_t)d.nkc * d.n_mt; break;
                case SETUP_ZERO_PAD: need = (j.n_words * 64 * (64 - (j.cols & 63)) + 2047) / 2048; if (need > 4096) need = 4096; break;
                default: need = (j.n_words + 2047) / 2048; if (need > 4096) need = 4096; break;   // 8 words per thread at least
            }
            if (need > grid_x) grid_x = need;
        }
        if (grid_x > 65535) {
            set_error("setup_jobs: grid too large");
            return LSTM_ERR_UNSUPPORTED;
        }
        KernelTimer timer(KC_AUX, s, 0.0, 0.0);
        LP_ONLY(dtype, T, hipLaunchKernelGGL(setup_jobs_kernel<T>, dim3((unsigned)grid_x, n), dim3(256), 0, s, a));
        LSTM_LAUNCH_CHECK();
    }
    return LSTM_OK;
}

int pack_rows(int dtype, const void *h, void *hpk, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_rows_kernel<T>, dim3(d.nkc, d.n_mt), dim3(256), 0, s, (const T *)h, (T *)hpk, B, H, d.nkc));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int step_forward_fused(int dtype, const void *hpk_prev, const void *Upk, const void *Ax, float *c_state, void *gates,
                       void *c_out, void *h_out, void *hpk_next, void *h_blk, int blk_ncb, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    FwdArgs a;
    a.hpk_prev = hpk_prev; a.Upk = Upk; a.Ax = Ax; a.c_state = c_state; a.gates = gates; a.c_out = c_out; a.h_out = h_out;
    a.xpk = nullptr; a.Wpk = nullptr; a.bias = nullptr; a.nkc2 = 0;
    a.hpk_next = hpk_next; a.h_blk = h_blk; a.blk_ncb = blk_ncb;
    a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc;
    if (narrow_cells(d, H)) {                                  // a few dozen workgroups: the latency-lean kernel
        WaveCell c{};
        c.hpk_prev = hpk_prev; c.Upk = Upk; c.Ax = Ax; c.c_state = c_state; c.gates = gates; c.c_out = c_out; c.h_out = h_out;
        c.hpk_next = hpk_next; c.h_blk = h_blk;
        return step_forward_wave(dtype, &c, 1, blk_ncb, B, H, s);
    }
    const bool wide = recurrent_wide(d);
    const int grid = d.n_mt * d.n_hb;
    // what the fused step has to move whatever the layout: U once; per unit the four pre-activations and c read, the four
    // gates, c and h written (26 bytes in a 16-bit type).  The extra copies of h_t this build writes for its own
    // consumers (packed, blocked) and the fp32 cell state are layout choices and are not counted.
    const double bh = (double)B * H;
    KernelTimer timer(KC_GEMM_STEP, s, 2.0 * B * 4.0 * H * H, 2.0 * 4.0 * H * H + 26.0 * bh);
    if (wide) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_forward_kernel<T, true>), dim3(grid), dim3(64), 0, s, a));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_forward_kernel<T, false>), dim3(grid), dim3(256), 0, s, a));
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

bool recurrent_wide_shape(int B, int H) { return recurrent_wide(recurrent_dims(B, H)); }

int pack_w_forward(int dtype, const void *W, void *Wpk, int H, int K, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(1, H);
    const int nkc = (K + SK - 1) / SK;
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_w_forward_kernel<T>, dim3(nkc, d.n_hb), dim3(256), 0, s, (const T *)W, (T *)Wpk, H, K, nkc));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int pack_rows_seq(int dtype, const void *x, void *xpk, int T_steps, int B, int K, int64_t dst_stride, hipStream_t s) {
    const int nkc = (K + SK - 1) / SK, n_mt = (B + TM - 1) / TM;
    if (T_steps < 1 || T_steps > 65535 || dst_stride < (int64_t)n_mt * nkc * A_CHUNK) {
        set_error("pack_rows_seq: bad sequence length %d or slot stride", T_steps);
        return LSTM_ERR_INVALID;
    }
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_rows_seq_kernel<T>, dim3(nkc, n_mt, T_steps), dim3(256), 0, s, (const T *)x, (T *)xpk, B, K, nkc,
                                         dst_stride));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

// as step_forward_fused, with the step's input projection done here: xpk = the step's input packed like h
// (in_width columns), Wpk = W packed by pack_w_forward, bias added in the epilogue
int step_forward_proj(int dtype, const void *hpk_prev, const void *Upk, const void *xpk, const void *Wpk, const void *bias, int in_width,
                      float *c_state, void *gates, void *c_out, void *h_out, void *hpk_next, void *h_blk, int blk_ncb, int B, int H,
                      hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (!xpk || !Wpk || !bias || in_width < 1) {
        set_error("step_forward_proj: null operand");
        return LSTM_ERR_INVALID;
    }
    FwdArgs a;
    a.hpk_prev = hpk_prev; a.Upk = Upk; a.Ax = nullptr; a.c_state = c_state; a.gates = gates; a.c_out = c_out; a.h_out = h_out;
    a.xpk = xpk; a.Wpk = Wpk; a.bias = bias; a.nkc2 = (in_width + SK - 1) / SK;
    a.hpk_next = hpk_next; a.h_blk = h_blk; a.blk_ncb = blk_ncb;
    a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc;
    const int grid = d.n_mt * d.n_hb;
    const double bh = (double)B * H;
    KernelTimer timer(KC_GEMM_STEP, s, 2.0 * B * 4.0 * H * ((double)H + in_width),
                      2.0 * (4.0 * H * ((double)H + in_width) + bh + (double)B * in_width) + 4.0 * bh +
                          2.0 * (4.0 * bh + bh + (h_blk ? 3.0 : 2.0) * bh) + 4.0 * bh);
    if (recurrent_wide(d)) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_forward_kernel<T, true>), dim3(grid), dim3(64), 0, s, a));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_forward_kernel<T, false>), dim3(grid), dim3(256), 0, s, a));
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

// the whole recurrence of a layer in one launch (lstm_rows_forward_kernel): thousands of rows, H <= 256
bool rows_forward_supported(int dtype, int B, int H, int in_width) {
    if (dtype != LSTM_DTYPE_FP16 && dtype != LSTM_DTYPE_BF16) return false;
    const RecurrentDims d = recurrent_dims(B, H);
    return H % 8 == 0 && recurrent_wide(d) && d.n_hb <= 8 && d.nkc <= 4 && in_width >= 1 && in_width <= 256;
}

int rows_forward(int dtype, const RowsForward &x, int in_width, int T, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (!rows_forward_supported(dtype, B, H, in_width) || !x.hseq || !x.xseq || !x.Upk || !x.Wpk || !x.bias || !x.c_state || !x.gates ||
        !x.c_out || !x.h_out || T < 1) {
        set_error("rows_forward: unsupported shape or null operand (B=%d H=%d)", B, H);
        return LSTM_ERR_INVALID;
    }
    RowsFwdArgs a;
    a.hseq = x.hseq; a.xseq = x.xseq; a.slot_h = x.slot_h; a.slot_x = x.slot_x; a.Upk = x.Upk; a.Wpk = x.Wpk; a.bias = x.bias;
    a.c_state = x.c_state; a.gates = x.gates; a.c_out = x.c_out; a.h_out = x.h_out; a.h_blk = x.h_blk; a.slot_blk = x.slot_blk;
    a.blk_ncb = x.blk_ncb; a.T = T; a.B = B; a.H = H; a.nkc = d.nkc; a.nkc2 = (in_width + SK - 1) / SK;
    a.in_width = in_width; a.all_h_out = x.all_h_out; a.write_hpk = x.write_hpk;
    const double bh = (double)B * H;
    // operands once: the weights per launch; per step x_t read, the gates, c_t and the copies of h_t written; c_0 / c_T in fp32
    const double h_copies = (x.all_h_out ? 1.0 : 0.0) + (x.write_hpk ? 1.0 : 0.0) + (x.h_blk ? 1.0 : 0.0);
    KernelTimer timer(KC_GEMM_STEP, s, (double)T * 2.0 * B * 4.0 * H * ((double)H + in_width),
                      2.0 * 4.0 * H * ((double)H + in_width) + 8.0 * bh +
                          (double)T * 2.0 * ((double)B * in_width + 4.0 * bh + bh + h_copies * bh));
    LP_ONLY(dtype, T_, hipLaunchKernelGGL(lstm_rows_forward_kernel<T_>, dim3(2 * d.n_mt), dim3(512), 0, s, a));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

// the whole BPTT recurrence of a layer in one launch (lstm_rows_backward_kernel): thousands of rows, H <= 256
int rows_backward_groups(int B) { return 2 * ((B + TM - 1) / TM); }

bool rows_backward_supported(int dtype, int B, int H) {
    if (dtype != LSTM_DTYPE_FP16 && dtype != LSTM_DTYPE_BF16) return false;
    const RecurrentDims d = recurrent_dims(B, H);
    return H % 8 == 0 && recurrent_wide(d) && d.n_hb <= 8 && d.nkc <= 4 && (rows_shape(d, H) || backward_slices(d) == 1);
}

int rows_backward(int dtype, const RowsBackward &x, int T, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    const uintptr_t all = (uintptr_t)x.UTpk | (uintptr_t)x.dh_above | (uintptr_t)x.gates | (uintptr_t)x.cs | (uintptr_t)x.dA | (uintptr_t)x.dAblk |
                          (uintptr_t)x.bias_partial;
    if (!rows_backward_supported(dtype, B, H) || !x.UTpk || !x.dh_above || !x.gates || !x.cs || (!x.dA && !x.dAblk) || T < 1 || all % 16 != 0) {
        set_error("rows_backward: unsupported shape, null or misaligned operand (B=%d H=%d)", B, H);
        return LSTM_ERR_INVALID;
    }
    RowsBwdArgs a;
    a.UTpk = x.UTpk; a.dh_above = x.dh_above; a.gates = x.gates; a.cs = x.cs; a.dA = x.dA; a.dAblk = x.dAblk; a.slot_blk = x.slot_blk;
    a.bias_partial = x.bias_partial;
    a.blk_ncb = x.blk_ncb; a.T = T; a.B = B; a.H = H; a.nkc = d.nkc;
    const double n = (double)B * H;
    // operands once: U per launch; per step the saved gates, c_t and the gradient from above read, dA written once per copy
    KernelTimer timer(KC_GEMM_STEP, s, (double)(T - 1) * 2.0 * n * 4.0 * H,
                      2.0 * 4.0 * H * H + (double)T * n * 2.0 * (6.0 + 4.0 * ((x.dA ? 1 : 0) + (x.dAblk ? 1 : 0))));
    LP_ONLY(dtype, T_, hipLaunchKernelGGL(lstm_rows_backward_kernel<T_>, dim3(2 * d.n_mt), dim3(512), 0, s, a));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int step_backward_gemm(int dtype, const void *dApk, const void *UTpk, float *partials, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    BwdArgs a;
    a.dApk = dApk; a.UTpk = UTpk; a.partials = partials;
    a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc; a.slices = backward_slices(d);
    const bool wide = recurrent_wide(d) && a.slices == 4;      // unsplit: the four wavefronts share the longer K range
    const int grid = d.n_mt * d.n_nt * a.slices;
    // U and dA read once, one fp32 dh written (the K-slice partials this build writes instead are a layout choice)
    KernelTimer timer(KC_GEMM_STEP, s, 2.0 * B * 4.0 * H * H, 2.0 * 4.0 * H * H + 12.0 * (double)B * H);
    if (wide) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_backward_gemm_kernel<T, true>), dim3(grid), dim3(64), 0, s, a));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_step_backward_gemm_kernel<T, false>), dim3(grid), dim3(256), 0, s, a));
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

bool step_backward_fused_supported(int dtype, int B, int H) {
    if (dtype != LSTM_DTYPE_FP16 && dtype != LSTM_DTYPE_BF16) return false;
    return H % 8 == 0 && backward_slices(recurrent_dims(B, H)) == 1;
}

int step_backward_fused(int dtype, const FusedBackwardCell &x, int blk_ncb, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    const uintptr_t all = (uintptr_t)x.dApk_next | (uintptr_t)x.UTpk | (uintptr_t)x.dh_above | (uintptr_t)x.gates | (uintptr_t)x.c_t |
                          (uintptr_t)x.c_prev | (uintptr_t)x.dc_state | (uintptr_t)x.dA | (uintptr_t)x.dApk | (uintptr_t)x.dAblk;
    if (!step_backward_fused_supported(dtype, B, H) || !x.gates || !x.c_t || !x.c_prev || !x.dc_state || !x.dApk || (!x.dA && !x.dAblk) ||
        (!x.dApk_next != !x.UTpk) || x.dApk_above || x.WTpk || !x.dh_above || (!x.first && !x.dApk_next) || all % 16 != 0) {
        set_error("step_backward_fused: unsupported shape or inconsistent / misaligned operands (B=%d H=%d)", B, H);
        return LSTM_ERR_INVALID;
    }
    FusedStepArgs a;
    a.c.dApk_next = x.dApk_next; a.c.UTpk = x.UTpk; a.c.dApk_above = nullptr; a.c.WTpk = nullptr; a.c.dh_above = x.dh_above;
    a.c.gates = x.gates; a.c.c_t = x.c_t; a.c.c_prev = x.c_prev; a.c.dc_state = x.dc_state; a.c.dA = x.dA; a.c.dApk = x.dApk;
    a.c.dAblk = x.dAblk; a.c.first = x.first;
    a.blk_ncb = blk_ncb; a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc;
    const double n = (double)B * H;
    KernelTimer timer(KC_GEMM_STEP, s, x.dApk_next ? 2.0 * n * 4.0 * H : 0.0,
                      (x.dApk_next ? 2.0 * (4.0 * H * H + 4.0 * n) : 0.0) + n * (8.0 + 2.0 * (7.0 + 4.0 * (1 + (x.dA ? 1 : 0) + (x.dAblk ? 1 : 0)))));
    LP_ONLY(dtype, T, hipLaunchKernelGGL(lstm_step_backward_fused_kernel<T>, dim3(d.n_mt * d.n_nt), dim3(256), 0, s, a));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int gates_backward_packed(int dtype, const void *dh_above, const float *partials, const void *gates, const void *c_t,
                          const void *c_prev, float *dc_state, void *dA, void *dApk, void *dAblk, int blk_ncb, int B, int H,
                          int first, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    const int64_t n = (int64_t)B * H;
    const uintptr_t all = (uintptr_t)dh_above | (uintptr_t)partials | (uintptr_t)gates | (uintptr_t)c_t | (uintptr_t)c_prev |
                          (uintptr_t)dc_state | (uintptr_t)dA | (uintptr_t)dApk | (uintptr_t)dAblk;
    const bool vec = H % 8 == 0 && all % 16 == 0;
    // 8 units per thread (16-byte accesses everywhere); 4 while that would leave fewer than two
    // wavefronts per SIMD on the chip (the kernel is latency-bound then)
    const int per_thread = !vec ? 1 : (n / 8 <= 256 * 256 * 2 ? 4 : 8);
    const int64_t items = n / per_thread;
    int blocks = (int)((items + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    // per unit: four fp32 partials and the cell gradient read, the cell gradient written, seven
    // 16-bit values read, four gate gradients written once per copy (packed, row-major, blocked)
    const int n_part = backward_slices(d);                      // as step_backward_gemm wrote them
    KernelTimer timer(KC_POINTWISE, s, 0.0, (double)n * (4.0 * n_part + 8.0 + 2.0 * (7.0 + 4.0 * (1 + (dA ? 1 : 0) + (dAblk ? 1 : 0)))));
#define LSTM_GATES_LAUNCH(W)                                                                                                   \
    LP_ONLY(dtype, T, hipLaunchKernelGGL((gates_backward_packed_kernel<T, W>), dim3(blocks), dim3(256), 0, s,                  \
                                         (const T *)dh_above, partials, (const T *)gates, (const T *)c_t, (const T *)c_prev,   \
                                         dc_state, (T *)dA, (T *)dApk, (T *)dAblk, blk_ncb, B, H, d.nkc, first, n_part))
    if (per_thread == 8) { LSTM_GATES_LAUNCH(8); }
    else if (per_thread == 4) { LSTM_GATES_LAUNCH(4); }
    else { LSTM_GATES_LAUNCH(1); }
#undef LSTM_GATES_LAUNCH
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int fused_backward_max_cells() { return FUSED_MAX_CELLS; }

// 16-byte accesses need H % 8 == 0; worth it while a cell is a few dozen workgroups
bool fused_backward_supported(int dtype, int B, int H) {
    if (dtype != LSTM_DTYPE_FP16 && dtype != LSTM_DTYPE_BF16) return false;
    return narrow_cells(recurrent_dims(B, H), H);
}

template <int NC>
static int launch_fused_backward(int dtype, const FusedBwdCell *cells, int n_cells, int blk_ncb, int B, int H, int nkc, hipStream_t s) {
    FusedBwdArgs<NC> w;
    for (int i = 0; i < NC; ++i) w.cell[i] = cells[i < n_cells ? i : 0];
    w.blk_ncb = blk_ncb; w.B = B; w.H = H; w.nkc = nkc;
    const int R = narrow_tile(B, H, n_cells);
    const dim3 grid((B + R - 1) / R, (H + R - 1) / R, n_cells);
    if (R == 16) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_fused_backward_kernel<T, 16, NC>), grid, dim3(256), 0, s, w));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_fused_backward_kernel<T, 32, NC>), grid, dim3(256), 0, s, w));
    }
    return LSTM_OK;
}

int backward_fused_wave(int dtype, const FusedBackwardCell *c, int n_cells, int blk_ncb, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (n_cells < 1 || n_cells > FUSED_MAX_CELLS || H % 8 != 0) {
        set_error("backward_fused_wave: %d cells (1..%d), H = %d (multiple of 8)", n_cells, FUSED_MAX_CELLS, H);
        return LSTM_ERR_INVALID;
    }
    FusedBwdCell cells[FUSED_MAX_CELLS];
    uintptr_t all = 0;
    double chunks = 0.0;
    for (int i = 0; i < n_cells; ++i) {
        const FusedBackwardCell &x = c[i];
        if (!x.gates || !x.c_t || !x.c_prev || !x.dc_state || !x.dApk || (!x.dA && !x.dAblk) || (!x.dApk_next != !x.UTpk) ||
            (!x.dApk_above != !x.WTpk) || (!x.dApk_above && !x.dh_above) || (!x.first && !x.dApk_next)) {
            set_error("backward_fused_wave: inconsistent operands in cell %d", i);
            return LSTM_ERR_INVALID;
        }
        all |= (uintptr_t)x.dApk_next | (uintptr_t)x.UTpk | (uintptr_t)x.dApk_above | (uintptr_t)x.WTpk | (uintptr_t)x.dh_above |
               (uintptr_t)x.gates | (uintptr_t)x.c_t | (uintptr_t)x.c_prev | (uintptr_t)x.dc_state | (uintptr_t)x.dA |
               (uintptr_t)x.dApk | (uintptr_t)x.dAblk;
        FusedBwdCell &o = cells[i];
        o.dApk_next = x.dApk_next; o.UTpk = x.UTpk; o.dApk_above = x.dApk_above; o.WTpk = x.WTpk; o.dh_above = x.dh_above;
        o.gates = x.gates; o.c_t = x.c_t; o.c_prev = x.c_prev; o.dc_state = x.dc_state; o.dA = x.dA; o.dApk = x.dApk;
        o.dAblk = x.dAblk; o.first = x.first;
        chunks += (x.dApk_next ? 1.0 : 0.0) + (x.dApk_above ? 1.0 : 0.0);
    }
    if (all % 16 != 0) {
        set_error("backward_fused_wave: operands must be 16-byte aligned");
        return LSTM_ERR_INVALID;
    }
    const double n = (double)B * H;
    // products: 2 B H 4H flops, operands once; gate arithmetic: as in the stand-alone kernel without the partials
    KernelTimer timer(KC_GEMM_STEP, s, chunks * 2.0 * n * 4.0 * H, chunks * 2.0 * (4.0 * H * H + 4.0 * n) + n_cells * n * (8.0 + 15.0 * 2.0));
    if (n_cells <= 2) { LSTM_TRY(launch_fused_backward<2>(dtype, cells, n_cells, blk_ncb, B, H, d.nkc, s)); }
    else if (n_cells <= 4) { LSTM_TRY(launch_fused_backward<4>(dtype, cells, n_cells, blk_ncb, B, H, d.nkc, s)); }
    else { LSTM_TRY(launch_fused_backward<FUSED_MAX_CELLS>(dtype, cells, n_cells, blk_ncb, B, H, d.nkc, s)); }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int wave_forward_max_cells() { return FUSED_MAX_CELLS; }   // step_forward_wave splits for the general kernel itself

template <int NC>
static int launch_narrow_forward(int dtype, const FwdArgs *cells, int n_cells, int B, int H, hipStream_t s) {
    NarrowFwdArgs<NC> w;
    for (int i = 0; i < NC; ++i) w.cell[i] = cells[i < n_cells ? i : 0];
    const int R = narrow_tile(B, H, n_cells);
    const dim3 grid((B + R - 1) / R, (H + R - 1) / R, n_cells);
    if (R == 16) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_narrow_forward_kernel<T, 16, NC>), grid, dim3(256), 0, s, w));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((lstm_narrow_forward_kernel<T, 32, NC>), grid, dim3(256), 0, s, w));
    }
    return LSTM_OK;
}

int step_forward_wave(int dtype, const WaveCell *cells, int n_cells, int blk_ncb, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (n_cells < 1 || n_cells > FUSED_MAX_CELLS) {
        set_error("step_forward_wave: %d cells (1..%d)", n_cells, FUSED_MAX_CELLS);
        return LSTM_ERR_INVALID;
    }
    FwdArgs args[FUSED_MAX_CELLS];
    uintptr_t all = 0;
    for (int i = 0; i < n_cells; ++i) {
        const WaveCell &c = cells[i];
        if (!c.hpk_prev || !c.Upk || !c.c_state || !c.gates || !c.c_out || !c.h_out || !c.hpk_next || (!c.Ax && (!c.xpk || !c.Wpk || !c.bias))) {
            set_error("step_forward_wave: null operand in cell %d", i);
            return LSTM_ERR_INVALID;
        }
        all |= (uintptr_t)c.hpk_prev | (uintptr_t)c.Upk | (uintptr_t)c.Ax | (uintptr_t)c.xpk | (uintptr_t)c.Wpk | (uintptr_t)c.bias |
               (uintptr_t)c.c_state | (uintptr_t)c.gates | (uintptr_t)c.c_out | (uintptr_t)c.h_out | (uintptr_t)c.hpk_next | (uintptr_t)c.h_blk;
        FwdArgs &a = args[i];
        a.hpk_prev = c.hpk_prev; a.Upk = c.Upk; a.Ax = c.Ax; a.xpk = c.xpk; a.Wpk = c.Wpk; a.bias = c.bias;
        a.c_state = c.c_state; a.gates = c.gates; a.c_out = c.c_out; a.h_out = c.h_out; a.hpk_next = c.hpk_next; a.h_blk = c.h_blk;
        a.blk_ncb = blk_ncb; a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc; a.nkc2 = d.nkc;
    }
    // per cell as in step_forward_fused; a cell that projects its input reads W and the packed
    // input instead of a ready-made projection
    auto work = [&](int first, int n, double &flops, double &bytes) {
        const double bh = (double)B * H;
        flops = bytes = 0.0;
        for (int i = first; i < first + n; ++i) {
            const bool proj = !cells[i].Ax;
            flops += 2.0 * B * 4.0 * H * H * (proj ? 2.0 : 1.0);
            bytes += 2.0 * 4.0 * H * H * (proj ? 2.0 : 1.0) + (proj ? 20.0 : 26.0) * bh;
        }
    };
    if (narrow_cells(d, H) && all % 16 == 0) {
        double flops, bytes;
        work(0, n_cells, flops, bytes);
        KernelTimer timer(KC_GEMM_STEP, s, flops, bytes);
        if (n_cells <= 2) { LSTM_TRY(launch_narrow_forward<2>(dtype, args, n_cells, B, H, s)); }
        else if (n_cells <= 4) { LSTM_TRY(launch_narrow_forward<4>(dtype, args, n_cells, B, H, s)); }
        else { LSTM_TRY(launch_narrow_forward<FUSED_MAX_CELLS>(dtype, args, n_cells, B, H, s)); }
        LSTM_LAUNCH_CHECK();
        return LSTM_OK;
    }
    // the general multi-cell kernel takes up to WAVE_MAX_CELLS cells per launch
    for (int first = 0; first < n_cells; first += WAVE_MAX_CELLS) {
        const int n = n_cells - first < WAVE_MAX_CELLS ? n_cells - first : WAVE_MAX_CELLS;
        WaveFwdArgs w;
        w.wgs_per_cell = d.n_mt * d.n_hb;
        for (int i = 0; i < WAVE_MAX_CELLS; ++i) w.cell[i] = args[first + (i < n ? i : 0)];
        double flops, bytes;
        work(first, n, flops, bytes);
        KernelTimer timer(KC_GEMM_STEP, s, flops, bytes);
        LP_ONLY(dtype, T, hipLaunchKernelGGL(lstm_wave_forward_kernel<T>, dim3(w.wgs_per_cell * n), dim3(256), 0, s, w));
        LSTM_LAUNCH_CHECK();
    }
    return LSTM_OK;
}

int wave_backward_max_gemms() { return WAVE_MAX_GEMMS; }
int wave_backward_max_gates() { return WAVE_MAX_GATES; }

int step_backward_gemm_wave(int dtype, const WaveGemm *g, int n, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (n < 1 || n > WAVE_MAX_GEMMS) {
        set_error("step_backward_gemm_wave: %d products (1..%d)", n, WAVE_MAX_GEMMS);
        return LSTM_ERR_INVALID;
    }
    WaveBwdGemmArgs w;
    for (int i = 0; i < WAVE_MAX_GEMMS; ++i) {
        const WaveGemm &c = g[i < n ? i : 0];
        if (!c.dApk || !c.Bpk || !c.partials) {
            set_error("step_backward_gemm_wave: null operand in product %d", i);
            return LSTM_ERR_INVALID;
        }
        w.dApk[i] = c.dApk; w.Bpk[i] = c.Bpk; w.partials[i] = c.partials;
    }
    w.B = B; w.H = H; w.n_mt = d.n_mt; w.nkc = d.nkc; w.wgs_per_cell = d.n_mt * d.n_nt * 4;
    KernelTimer timer(KC_GEMM_STEP, s, n * 2.0 * B * 4.0 * H * H, n * (2.0 * 4.0 * H * H + 12.0 * (double)B * H));
    LP_ONLY(dtype, T, hipLaunchKernelGGL(lstm_wave_backward_gemm_kernel<T>, dim3(w.wgs_per_cell * n), dim3(256), 0, s, w));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int gates_backward_wave(int dtype, const WaveGates *c, int n_cells, int blk_ncb, int B, int H, hipStream_t s, int n_part) {
    const RecurrentDims d = recurrent_dims(B, H);
    if (n_cells < 1 || n_cells > WAVE_MAX_GATES) {
        set_error("gates_backward_wave: %d cells (1..%d)", n_cells, WAVE_MAX_GATES);
        return LSTM_ERR_INVALID;
    }
    const int64_t n = (int64_t)B * H;
    uintptr_t all = 0;
    WaveGateArgs w;
    for (int i = 0; i < WAVE_MAX_GATES; ++i) {
        const WaveGates &x = c[i < n_cells ? i : 0];
        if (!x.gates || !x.c_t || !x.c_prev || !x.dc_state || !x.dApk || (!x.first && !x.partials) || (!x.dh_above && !x.above4)) {
            set_error("gates_backward_wave: null operand in cell %d", i);
            return LSTM_ERR_INVALID;
        }
        all |= (uintptr_t)x.dh_above | (uintptr_t)x.above4 | (uintptr_t)x.partials | (uintptr_t)x.gates | (uintptr_t)x.c_t |
               (uintptr_t)x.c_prev | (uintptr_t)x.dc_state | (uintptr_t)x.dA | (uintptr_t)x.dApk | (uintptr_t)x.dAblk;
        WaveGateCell &o = w.cell[i];
        o.dh_above = x.dh_above; o.above4 = x.above4; o.partials = x.partials; o.gates = x.gates; o.c_t = x.c_t; o.c_prev = x.c_prev;
        o.dc_state = x.dc_state; o.dA = x.dA; o.dApk = x.dApk; o.dAblk = x.dAblk; o.first = x.first;
    }
    const bool vec = H % 8 == 0 && all % 16 == 0;
    const int64_t items = vec ? n / 8 : n;
    int blocks = (int)((items + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    w.blk_ncb = blk_ncb; w.B = B; w.H = H; w.nkc = d.nkc; w.blocks_per_cell = blocks; w.n_part = n_part;
    // per unit and cell: the fp32 partial sums and the cell gradient read, the cell gradient written, seven 16-bit values
    // read, four gate gradients written once per copy that exists (packed always; row-major, blocked)
    double copies = 0.0;
    for (int i = 0; i < n_cells; ++i) copies += 1.0 + (c[i].dA ? 1.0 : 0.0) + (c[i].dAblk ? 1.0 : 0.0);
    KernelTimer timer(KC_POINTWISE, s, 0.0, (double)n * (n_cells * (4.0 * n_part + 8.0 + 7.0 * 2.0) + copies * 4.0 * 2.0));
    if (vec) {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((wave_gates_backward_kernel<T, 8>), dim3(blocks * n_cells), dim3(256), 0, s, w));
    } else {
        LP_ONLY(dtype, T, hipLaunchKernelGGL((wave_gates_backward_kernel<T, 1>), dim3(blocks * n_cells), dim3(256), 0, s, w));
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace lstm
