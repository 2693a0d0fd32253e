// Launch wrappers of the pointwise / reduction / optimiser kernels (internal).
#pragma once
#include "common.h"

namespace lstm {

// fill n 32-bit words with `value`
int fill_u32(void *dst, uint32_t value, int64_t n_words, hipStream_t s);

// state set-up of one layer: h slot 0 / c slot 0 of the saved sequences and
// the running fp32 cell state, from h0/c0 (null = zeros)
int init_state(int dtype, const void *h0, const float *c0, void *h_slot0, void *c_slot0, float *c_state, int64_t n,
               hipStream_t s);

// one time step of the gate non-linearities and the cell/hidden update
//   A       fp32 [B,4H] pre-activations (W x + U h + b)
//   c_state fp32 [B,H]  in: c_{t-1}, out: c_t
//   gates   lp   [B,4H] out: i,f,g,o
//   c_out,h_out lp [B,H]
int gates_forward(int dtype, const float *A, float *c_state, void *gates, void *c_out, void *h_out, int B, int H,
                  hipStream_t s);

// one time step of BPTT through the gates
//   dh_above lp [B,H] (null = 0), dh_rec fp32 [n_rec][B,H] partial sums (null = 0)
//   gates lp [B,4H], c_t / c_prev lp [B,H]
//   dc_state fp32 [B,H]: in dc carried from t+1 (ignored when first != 0), out dc for t-1
//   dA lp [B,4H] out
int gates_backward(int dtype, const void *dh_above, const float *dh_rec, const void *gates, const void *c_t,
                   const void *c_prev, float *dc_state, void *dA, int B, int H, int first, int n_rec, hipStream_t s);

// out[C,R] = in[R,C]^T for lp elements
int transpose_lp(int dtype, const void *in, int64_t ld_in, void *out, int64_t ld_out, int R, int C, hipStream_t s);

// out_lp[c] = scale * sum_r w[r] * in[r,c]   (w null = 1; scale_dev null = 1)
// partial: fp32 [chunks, C] workspace with chunks = colsum_chunks(R)
int colsum_chunks(int R);
// Several workers (rows interleaved in segments of `seg` rows per time step, see RowSeg in
// pointwise.hip): R rows per worker, one result per worker out_stride elements apart,
// partial then holds workers * chunks * C floats.
int colsum(int dtype, const void *in, int64_t ld, int R, int C, const float *row_w, const float *scale_dev,
           float *partial, void *out_lp, hipStream_t s, int workers = 1, int seg = 0, int64_t out_stride = 0);

// the same sums (no weights, no scale) of a 16-bit tensor stored in 64x64 blocks with ncb column
// blocks per row block; partial holds workers * colsum_blocked_chunks(R) * C floats.  Several workers:
// R rows each, laid out as consecutive segments of seg_rows rows (a multiple of 64) per worker that
// repeat every workers * seg_rows rows; worker w's sums go to out_lp + w * out_stride.
// packed = 1: every 64x64 block holds its elements in MFMA-fragment order (packed.h, two 32-row blocks).
int colsum_blocked_chunks(int R);
// out_lp[w * out_stride + c] = sum over k < chunks of partial[(w * chunks + k) * C + c], w < workers (16-bit types)
int colsum_finish(int dtype, const float *partial, int chunks, int C, void *out_lp, hipStream_t s, int workers, int64_t out_stride);
int colsum_blocked(int dtype, const void *blk, int ncb, int R, int C, float *partial, void *out_lp, hipStream_t s, int workers = 1,
                   int seg_rows = 0, int64_t out_stride = 0, int packed = 0);

// head forward: z = h.w + b per row; loss partial sums; dzu = dloss/dz (unscaled, already / M)
int head_loss_blocks(int rows);
int head_forward(int dtype, int head, const void *h_top, const void *w, const void *b, const float *targets, int rows,
                 int H, int M_total, float *dzu, float *partial, float *loss, hipStream_t s, int workers = 1, int seg = 0);
// dh[row,:] = scale * dzu[row] * w, zeroed where relu_of (same shape, may be null) is not positive
int head_backward_dh(int dtype, const float *dzu, const void *w, const float *scale_dev, const void *relu_of, void *dh,
                     int rows, int H, hipStream_t s);
// a = max(a, 0) element-wise
int relu_inplace(int dtype, void *a, int64_t n, hipStream_t s);
// db_head = scale * sum dzu
int head_backward_bias(int dtype, const float *dzu, const float *scale_dev, int rows, void *out_lp, hipStream_t s,
                       int workers = 1, int seg = 0, int64_t out_stride = 0);

// embedding: X[row,:] = E[clamp(ids[row]),:]
int embed_gather(int dtype, const int32_t *ids, const void *E, void *X, int rows, int V, int D, hipStream_t s);
// dE32[ids[row],:] += dX[row,:]  (fp32 atomics), then dE_lp = cast(dE32)
int embed_scatter_add(int dtype, const int32_t *ids, const void *dX, float *dE32, int rows, int V, int D, hipStream_t s);
int cast_f32_to_lp(int dtype, const float *in, void *out, int64_t n, hipStream_t s);
// copy final states out
int copy_state(int dtype, const void *h_src, const float *c_src, void *h_dst, float *c_dst, int64_t n, hipStream_t s);

// ---- fused per-time-step kernels (half / bfloat16 only), operands in packed tile order
struct RecurrentDims {
    int n_mt, n_hb, n_nt, nkc;          // batch tiles of 64, hidden blocks of 32, unit tiles of 128, K chunks of 64
    size_t upk_elems, utpk_elems;        // packed U for the forward / backward kernels
    size_t hpk_elems, dapk_elems;        // packed h (one step) / packed dA (one step)
    size_t partial_bytes;                // fp32 [4][B,H] recurrent partial sums
};
RecurrentDims recurrent_dims(int B, int H);
int pack_u_forward(int dtype, const void *U, void *Upk, int H, hipStream_t s);
int pack_u_backward(int dtype, const void *U, void *UTpk, int H, hipStream_t s);
// hpk = packed copy of row-major h [B,H] (h null = zeros); also clears the padding
int pack_rows(int dtype, const void *h, void *hpk, int B, int H, hipStream_t s);
// several packing jobs and zero fills in one launch (16-bit types)
enum { SETUP_PACK_U_FORWARD = 0, SETUP_PACK_U_BACKWARD = 1, SETUP_PACK_ROWS = 2, SETUP_ZERO = 3, SETUP_ZERO_PAD = 4 };
struct SetupJob {
    int kind;
    const void *src;      // U / W [4H,H], or h [B,H] (null: zeros) for SETUP_PACK_ROWS; unused for the fills
    void *dst;
    int64_t n_words;      // SETUP_ZERO: 32-bit words to clear; SETUP_ZERO_PAD: row blocks of the blocked tensor
    int ncb, cols;        // SETUP_ZERO_PAD: column blocks per row block, valid columns C (C % 64 != 0): the columns
                          // C % 64 .. 63 of the last column block of every row block are cleared (16-bit elements)
};
int setup_jobs(int dtype, const SetupJob *jobs, int n_jobs, int B, int H, hipStream_t s);
// forward: gates, c, h of one step from packed h_prev, packed U and the step's input projection Ax (lp, bias included);
// h_blk (nullable): first block row of this time slot in a 64x64-blocked copy of the hidden sequence
int step_forward_fused(int dtype, const void *hpk_prev, const void *Upk, const void *Ax, float *c_state, void *gates,
                       void *c_out, void *h_out, void *hpk_next, void *h_blk, int blk_ncb, int B, int H, hipStream_t s);
// The same with the step's input projection done in the kernel (large batches of narrow layers, where a
// whole-sequence projection is bound by writing and re-reading its [T*B, 4H] result): W packed for an
// input width K, a sequence [T, B, K] packed step by step (slot stride in elements).
bool recurrent_wide_shape(int B, int H);
// a layer's whole forward recurrence in one launch; operands as step_forward_proj takes them, per time slot
struct RowsForward {
    const void *hseq;          // packed h slots: slot 0 = h_0 (in), slot t + 1 = h_t (out)
    const void *xseq;          // packed input slots
    int64_t slot_h, slot_x;    // elements per slot
    const void *Upk, *Wpk, *bias;
    float *c_state;            // [B,H]: c_0 in, c_T out
    void *gates;               // [T][B,4H]
    void *c_out, *h_out;       // step 0's [B,H] (slot 1 of the saved sequences)
    void *h_blk;               // step 0's blocked slot, or null
    int64_t slot_blk;
    int blk_ncb;
    int all_h_out;             // 0: only h_T is written to h_out
    int write_hpk;             // 0: the packed h_t slots (a layer above reads them as its input) are not written
};
// a layer's whole BPTT recurrence in one launch: dA_t for every step from the saved activations and dh from above
struct RowsBackward {
    const void *UTpk;          // packed U^T (pack_u_backward)
    const void *dh_above;      // lp [T][B,H]
    const void *gates;         // lp [T][B,4H]
    const void *cs;            // lp [T+1][B,H] saved cell states (slot 0 = c_0)
    void *dA;                  // lp [T][B,4H] row-major out, or null
    void *dAblk;               // blocked out (slot_blk elements per time step), or null
    int64_t slot_blk;
    int blk_ncb;
    float *bias_partial;       // out or null: [rows_backward_groups(B)][4H] column sums of dA (fp32, before its rounding to
                               // 16 bits) over all T steps and the 32 rows of group i = rows 32 i .. 32 i + 31: the bias
                               // gradient's parts
};
int rows_backward_groups(int B);
bool rows_backward_supported(int dtype, int B, int H);
int rows_backward(int dtype, const RowsBackward &x, int T, int B, int H, hipStream_t s);
bool rows_forward_supported(int dtype, int B, int H, int in_width);
int rows_forward(int dtype, const RowsForward &x, int in_width, int T, int B, int H, hipStream_t s);
int pack_w_forward(int dtype, const void *W, void *Wpk, int H, int K, hipStream_t s);
int pack_rows_seq(int dtype, const void *x, void *xpk, int T_steps, int B, int K, int64_t dst_stride, hipStream_t s);
int step_forward_proj(int dtype, const void *hpk_prev, const void *Upk, const void *xpk, const void *Wpk, const void *bias, int in_width,
                      float *c_state, void *gates, void *c_out, void *h_out, void *hpk_next, void *h_blk, int blk_ncb, int B, int H,
                      hipStream_t s);
// backward: partials[q][B,H] = dA_next[:, gate q rows] * U[gate q rows, :] for q = 0..3
int step_backward_gemm(int dtype, const void *dApk, const void *UTpk, float *partials, int B, int H, hipStream_t s);
// BPTT through the gates; dA written row-major, packed, and (dAblk non-null: first block row of the time slot) 64x64-blocked
int gates_backward_packed(int dtype, const void *dh_above, const float *partials, const void *gates, const void *c_t,
                          const void *c_prev, float *dc_state, void *dA, void *dApk, void *dAblk, int blk_ncb, int B, int H,
                          int first, hipStream_t s);

// Up to wave_forward_max_cells() independent (layer, time) cells in one launch.  A cell either
// takes its input projection ready-made (Ax) or computes it from the packed h_t of the layer
// below (xpk), W packed like U (Wpk) and the bias.
struct WaveCell {
    const void *hpk_prev, *Upk, *Ax, *xpk, *Wpk, *bias;
    float *c_state;
    void *gates, *c_out, *h_out, *hpk_next, *h_blk;
};
// backward along anti-diagonals: several per-step products / several cells' gate arithmetic per launch
struct WaveGemm {
    const void *dApk, *Bpk;   // packed dA_t and packed U^T (or W^T) of its layer
    float *partials;          // fp32 [4][B,H] out
};
struct WaveGates {
    const void *dh_above;     // lp [B,H] or null
    const float *above4;      // fp32 [4][B,H] (dA_t W of the layer above) or null
    const float *partials;    // fp32 [4][B,H] (dA_{t+1} U), unused when first
    const void *gates, *c_t, *c_prev;
    float *dc_state;
    void *dA, *dApk, *dAblk;
    int first;
};
int wave_backward_max_gemms();
int wave_backward_max_gates();
int step_backward_gemm_wave(int dtype, const WaveGemm *g, int n, int B, int H, hipStream_t s);
// n_part: K-slice partials per cell behind WaveGates::partials (4: one per gate; 2: step_backward_gemm_tile's)
int gates_backward_wave(int dtype, const WaveGates *c, int n_cells, int blk_ncb, int B, int H, hipStream_t s, int n_part = 4);
// One BPTT cell done in a single launch (narrow layers): the recurrent products and the gate
// arithmetic together.  dApk_next / UTpk: packed dA_{t+1} and U^T of the cell's layer (null at the
// last time step); dApk_above / WTpk: packed dA_t and W^T of the layer above (null for the top
// layer, whose gradient arrives in dh_above).
struct FusedBackwardCell {
    const void *dApk_next, *UTpk, *dApk_above, *WTpk;
    const void *dh_above;     // lp [B,H] or null
    const void *gates, *c_t, *c_prev;
    float *dc_state;
    void *dA, *dApk, *dAblk;  // dA row-major (nullable), packed (the next step's operand), blocked (nullable)
    int first;
};
// one BPTT step of one layer in a single launch on the large-batch tiles (dApk_above / WTpk must be null)
bool step_backward_fused_supported(int dtype, int B, int H);
int step_backward_fused(int dtype, const FusedBackwardCell &c, int blk_ncb, int B, int H, hipStream_t s);
int fused_backward_max_cells();
bool fused_backward_supported(int dtype, int B, int H);
int backward_fused_wave(int dtype, const FusedBackwardCell *c, int n_cells, int blk_ncb, int B, int H, hipStream_t s);
// The same per-cell work on the wide-layer kernels (recurrent_tile.hip): H a multiple of 128, batch a multiple
// of 64, 16-bit types; every cell takes a ready-made input projection (Ax).  Up to tile_max_cells() per launch.
bool tile_kernels_supported(int dtype, int B, int H);
int tile_max_cells();
int step_forward_tile(int dtype, const WaveCell *cells, int n_cells, int blk_ncb, int B, int H, hipStream_t s);
// partials[q][B,H], q < tile_backward_slices(): the contraction over the rows of the gates of slice q
int tile_backward_slices();
int step_backward_gemm_tile(int dtype, const WaveGemm *g, int n, int B, int H, hipStream_t s);
int wave_forward_max_cells();
int step_forward_wave(int dtype, const WaveCell *cells, int n_cells, int blk_ncb, int B, int H, hipStream_t s);

}  // namespace lstm
