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
// in plain row-major order for the whole-sequence GEMMs).
#include "kernels.h"

namespace lstm {
namespace {

constexpr int TM = 64;                 // batch rows per workgroup
constexpr int NBLK = 4;                // 32-row B blocks per workgroup
constexpr int TN = NBLK * 32;          // B rows per workgroup
constexpr int SK = 64;                 // K elements per packed chunk
constexpr int NLD_A = TM * SK / 8 / 64;   // 16-byte loads per lane and chunk, A operand (8)
constexpr int NLD_B = TN * SK / 8 / 64;   // same, B operand (16)
constexpr int RED_FLOATS = 8 * 16 * 64;   // one wavefront's 8 accumulator blocks
constexpr int A_CHUNK = TM * SK;       // elements of one packed A block
constexpr int B_CHUNK = TN * SK;       // elements of one packed B block

// offset of element (row, kk) inside a packed chunk whose rows form `nblk` blocks of 32
__host__ __device__ inline int frag_offset(int row, int kk, int nblk) {
    const int blk = row >> 5, r = row & 31, ks = kk >> 4, half = (kk >> 3) & 1, j = kk & 7;
    return (((ks * nblk + blk) * 64) + half * 32 + r) * 8 + j;
}

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
                                                v16f (&acc)[2][NBLK]) {
    const int nst = c1 - c0;
    if (nst <= 0) return;
    rot %= nst;
    auto pa = [&](int s) {
        int ss = s + rot;
        if (ss >= nst) ss -= nst;
        return reinterpret_cast<const u32x4 *>(Apk + (int64_t)(c0 + ss) * A_CHUNK);
    };
    auto pb = [&](int s) {
        int ss = s + rot;
        if (ss >= nst) ss -= nst;
        return reinterpret_cast<const u32x4 *>(Bpk + (int64_t)(c0 + ss) * B_CHUNK);
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
    float *mine = red + wave * RED_FLOATS;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBLK; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[((mb * NBLK + nb) * 16 + r) * 64 + lane] = acc[mb][nb][r];
    __syncthreads();
    const int mb = wave >> 1, rh = (wave & 1) * 8;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr)
#pragma unroll
        for (int nb = 0; nb < NBLK; ++nb) {
            const int idx = ((mb * NBLK + nb) * 16 + rh + rr) * 64 + lane;
            out[rr][nb] = (red[idx] + red[RED_FLOATS + idx]) + (red[2 * RED_FLOATS + idx] + red[3 * RED_FLOATS + idx]);
        }
}

// linear tile index with workgroups of one XCD (id % 8) on neighbouring tiles,
// so that tiles sharing B rows share that XCD's L2
__device__ __forceinline__ int xcd_swizzle(int wg, int total) {
    return (total % 8 == 0) ? (wg % 8) * (total / 8) + wg / 8 : wg;
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
    const float *Ax;       // fp32 [B,4H], input projection + bias of this step
    float *c_state;        // fp32 [B,H] in/out
    void *gates;           // lp [B,4H] out
    void *c_out;           // lp [B,H] out
    void *h_out;           // lp [B,H] out (row-major)
    void *hpk_next;        // packed h_t out
    int B, H, n_mt, nkc;
};

template <typename T>
__global__ __launch_bounds__(256) void lstm_step_forward_kernel(FwdArgs a) {
    __shared__ __attribute__((aligned(16))) float smem[4 * RED_FLOATS];   // 128 KB: cross-wavefront reduction
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = xcd_swizzle(blockIdx.x, gridDim.x);
    const int mt = tile % a.n_mt, hb = tile / a.n_mt;
    const int m0 = mt * TM, j0 = hb * 32;
    const int H = a.H, G = 4 * a.H;
    const int cpw = (a.nkc + 3) / 4;                       // chunks per wavefront
    const int c0 = min(a.nkc, wave * cpw), c1 = min(a.nkc, c0 + cpw);
    v16f acc[2][NBLK];
    zero_acc(acc);
    packed_mainloop<T>(reinterpret_cast<const uint16_t *>(a.hpk_prev) + (int64_t)mt * a.nkc * A_CHUNK,
                       reinterpret_cast<const uint16_t *>(a.Upk) + (int64_t)hb * a.nkc * B_CHUNK, c0, c1, (int)blockIdx.x,
                       lane, acc);
    float pre[8][NBLK];
    reduce_waves(smem, wave, lane, acc, pre);

    const int mb = wave >> 1, rh = (wave & 1) * 8;
    const int j = j0 + (lane & 31);
    if (j >= H) return;
    T *gates = reinterpret_cast<T *>(a.gates);
    T *c_out = reinterpret_cast<T *>(a.c_out);
    T *h_out = reinterpret_cast<T *>(a.h_out);
    T *hpk = reinterpret_cast<T *>(a.hpk_next) + ((int64_t)mt * a.nkc + (j >> 6)) * A_CHUNK;
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int r = rh + rr;
        const int rl = mb * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int row = m0 + rl;
        if (row >= a.B) continue;
        const float *ax = a.Ax + (int64_t)row * G + j;
        const float gi = sigmoidf_dev(pre[rr][0] + ax[0]);
        const float gf = sigmoidf_dev(pre[rr][1] + ax[H]);
        const float gg = tanhf_dev(pre[rr][2] + ax[2 * H]);
        const float go = sigmoidf_dev(pre[rr][3] + ax[3 * H]);
        const int64_t e = (int64_t)row * H + j;
        const float c = gf * a.c_state[e] + gi * gg;
        const T h = Lp<T>::from_f(go * tanhf_dev(c));
        a.c_state[e] = c;
        T *gr = gates + (int64_t)row * G + j;
        gr[0] = Lp<T>::from_f(gi);
        gr[H] = Lp<T>::from_f(gf);
        gr[2 * H] = Lp<T>::from_f(gg);
        gr[3 * H] = Lp<T>::from_f(go);
        c_out[e] = Lp<T>::from_f(c);
        h_out[e] = h;
        hpk[frag_offset(rl, j & 63, 2)] = h;
    }
}

// ---------------------------------------------------------------- backward
struct BwdArgs {
    const void *dApk;      // packed dA_{t+1}: [n_mt][4][nkc][64][64]
    const void *UTpk;      // packed U^T: [n_nt][4][nkc][128][64]
    float *partials;       // fp32 [4][B,H] out: one K-slice (gate) each
    int B, H, n_mt, nkc;
};

// partial[q][b, j] = sum over the rows k of gate q of dA_next[b, k] * U[k, j]
template <typename T>
__global__ __launch_bounds__(256) void lstm_step_backward_gemm_kernel(BwdArgs a) {
    __shared__ __attribute__((aligned(16))) float smem[4 * RED_FLOATS];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lin = xcd_swizzle(blockIdx.x, gridDim.x);
    const int q = lin & 3, tile = lin >> 2;
    const int mt = tile % a.n_mt, nt = tile / a.n_mt;
    const int m0 = mt * TM, n0 = nt * TN;
    const int H = a.H;
    const int cpw = (a.nkc + 3) / 4;
    const int c0 = min(a.nkc, wave * cpw), c1 = min(a.nkc, c0 + cpw);
    v16f acc[2][NBLK];
    zero_acc(acc);
    packed_mainloop<T>(reinterpret_cast<const uint16_t *>(a.dApk) + ((int64_t)mt * 4 + q) * a.nkc * A_CHUNK,
                       reinterpret_cast<const uint16_t *>(a.UTpk) + ((int64_t)nt * 4 + q) * a.nkc * B_CHUNK, c0, c1,
                       (int)blockIdx.x, lane, acc);
    float sum[8][NBLK];
    reduce_waves(smem, wave, lane, acc, sum);
    const int mb = wave >> 1, rh = (wave & 1) * 8;
    float *part = a.partials + (int64_t)q * a.B * H;
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
}

// BPTT through the gates of one step; sums the four recurrent partials, writes
// dA row-major (for the whole-sequence GEMMs) and packed (A operand of the next
// recurrent GEMM).
template <typename T>
__global__ __launch_bounds__(256) void gates_backward_packed_kernel(const T *dh_above, const float *partials, const T *gates,
                                                                    const T *c_t, const T *c_prev, float *dc_state, T *dA,
                                                                    T *dApk, int B, int H, int nkc, int first) {
    const int64_t n = (int64_t)B * H;
    const int G = 4 * H;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(e / H), j = (int)(e % H);
        const T *gr = gates + (int64_t)b * G + j;
        const float i = Lp<T>::to_f(gr[0]), f = Lp<T>::to_f(gr[H]);
        const float g = Lp<T>::to_f(gr[2 * H]), o = Lp<T>::to_f(gr[3 * H]);
        const float tc = tanhf_dev(Lp<T>::to_f(c_t[e]));
        float dh = Lp<T>::to_f(dh_above[e]);
        float dcr = 0.0f;
        if (!first) {
            dh += (partials[e] + partials[n + e]) + (partials[2 * n + e] + partials[3 * n + e]);
            dcr = dc_state[e];
        }
        const float d_o = dh * tc;
        const float dc = dcr + dh * o * (1.0f - tc * tc);
        const float di = dc * g, dg = dc * i, df = dc * Lp<T>::to_f(c_prev[e]);
        dc_state[e] = dc * f;
        const T v0 = Lp<T>::from_f(di * i * (1.0f - i));
        const T v1 = Lp<T>::from_f(df * f * (1.0f - f));
        const T v2 = Lp<T>::from_f(dg * (1.0f - g * g));
        const T v3 = Lp<T>::from_f(d_o * o * (1.0f - o));
        T *da = dA + (int64_t)b * G + j;
        da[0] = v0; da[H] = v1; da[2 * H] = v2; da[3 * H] = v3;
        // packed: [b / 64][gate][j / 64] chunk, fragment order inside
        T *pk = dApk + (((int64_t)(b >> 6) * 4) * nkc + (j >> 6)) * A_CHUNK + frag_offset(b & 63, j & 63, 2);
        const int64_t gs = (int64_t)nkc * A_CHUNK;
        pk[0] = v0; pk[gs] = v1; pk[2 * gs] = v2; pk[3 * gs] = v3;
    }
}

// ---------------------------------------------------------------- packing
// chunk (hb, kc) of Upk, row g*32 + r, column kk = U[g*H + hb*32 + r][kc*64 + kk], zero outside
template <typename T>
__global__ __launch_bounds__(256) void pack_u_forward_kernel(const T *U, T *Upk, int H, int nkc) {
    const int hb = blockIdx.y, kc = blockIdx.x;
    T *dst = Upk + ((int64_t)hb * nkc + kc) * B_CHUNK;
    for (int v = threadIdx.x; v < B_CHUNK; v += 256) {
        const int row = v >> 6, kk = v & 63;
        const int g = row >> 5, r = row & 31;
        const int unit = hb * 32 + r, k = kc * 64 + kk;
        dst[frag_offset(row, kk, NBLK)] = (unit < H && k < H) ? U[((int64_t)g * H + unit) * H + k] : Lp<T>::from_f(0.0f);
    }
}
// chunk (nt, q, kc) of UTpk, row r, column kk = U[q*H + kc*64 + kk][nt*128 + r], zero outside
template <typename T>
__global__ __launch_bounds__(256) void pack_u_backward_kernel(const T *U, T *UTpk, int H, int nkc) {
    __shared__ T tile[64][TN + 2];
    const int nt = blockIdx.z, q = blockIdx.y, kc = blockIdx.x;
    // read U rows (k) x columns (units) coalesced along units, write transposed
    for (int v = threadIdx.x; v < 64 * TN; v += 256) {
        const int kk = v / TN, r = v % TN;
        const int k = kc * 64 + kk, unit = nt * TN + r;
        tile[kk][r] = (k < H && unit < H) ? U[((int64_t)q * H + k) * H + unit] : Lp<T>::from_f(0.0f);
    }
    __syncthreads();
    T *dst = UTpk + (((int64_t)nt * 4 + q) * nkc + kc) * B_CHUNK;
    for (int v = threadIdx.x; v < B_CHUNK; v += 256) dst[frag_offset(v >> 6, v & 63, NBLK)] = tile[v & 63][v >> 6];
}
// chunk (mt, kc) of hpk, row, column kk = h[mt*64 + row][kc*64 + kk] (null h = 0), zero outside
template <typename T>
__global__ __launch_bounds__(256) void pack_rows_kernel(const T *h, T *hpk, int B, int H, int nkc) {
    const int mt = blockIdx.y, kc = blockIdx.x;
    T *dst = hpk + ((int64_t)mt * nkc + kc) * A_CHUNK;
    for (int v = threadIdx.x; v < A_CHUNK; v += 256) {
        const int row = mt * 64 + (v >> 6), k = kc * 64 + (v & 63);
        dst[frag_offset(v >> 6, v & 63, 2)] = (h && row < B && k < H) ? h[(int64_t)row * H + k] : Lp<T>::from_f(0.0f);
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

int pack_rows(int dtype, const void *h, void *hpk, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(pack_rows_kernel<T>, dim3(d.nkc, d.n_mt), dim3(256), 0, s, (const T *)h, (T *)hpk, B, H, d.nkc));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int step_forward_fused(int dtype, const void *hpk_prev, const void *Upk, const float *Ax, float *c_state, void *gates,
                       void *c_out, void *h_out, void *hpk_next, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    FwdArgs a;
    a.hpk_prev = hpk_prev; a.Upk = Upk; a.Ax = Ax; a.c_state = c_state; a.gates = gates; a.c_out = c_out; a.h_out = h_out;
    a.hpk_next = hpk_next;
    a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc;
    const int grid = d.n_mt * d.n_hb;
    KernelTimer timer(KC_GEMM_STEP, s, 2.0 * B * 4.0 * H * H, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(lstm_step_forward_kernel<T>, dim3(grid), dim3(256), 0, s, a));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int step_backward_gemm(int dtype, const void *dApk, const void *UTpk, float *partials, int B, int H, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    BwdArgs a;
    a.dApk = dApk; a.UTpk = UTpk; a.partials = partials;
    a.B = B; a.H = H; a.n_mt = d.n_mt; a.nkc = d.nkc;
    const int grid = d.n_mt * d.n_nt * 4;
    KernelTimer timer(KC_GEMM_STEP, s, 2.0 * B * 4.0 * H * H, 0.0);
    LP_ONLY(dtype, T, hipLaunchKernelGGL(lstm_step_backward_gemm_kernel<T>, dim3(grid), dim3(256), 0, s, a));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int gates_backward_packed(int dtype, const void *dh_above, const float *partials, const void *gates, const void *c_t,
                          const void *c_prev, float *dc_state, void *dA, void *dApk, int B, int H, int first, hipStream_t s) {
    const RecurrentDims d = recurrent_dims(B, H);
    const int64_t n = (int64_t)B * H;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    KernelTimer timer(KC_POINTWISE, s, 0.0, (double)n * (16.0 + 8.0 + 15.0 * 2.0));
    LP_ONLY(dtype, T, hipLaunchKernelGGL(gates_backward_packed_kernel<T>, dim3(blocks), dim3(256), 0, s, (const T *)dh_above,
                                         partials, (const T *)gates, (const T *)c_t, (const T *)c_prev, dc_state, (T *)dA,
                                         (T *)dApk, B, H, d.nkc, first));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace lstm
