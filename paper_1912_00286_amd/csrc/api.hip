// C ABI entry points for the forward and backward halves of the training
// step, plus the layout bookkeeping (parameter offsets, workspace plan).
// Host code only orchestrates: every arithmetic step runs in a HIP kernel.
#include <stdarg.h>
#include <stdio.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "kernels.h"

namespace lstm {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

namespace {

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Everything derived from a config: parameter offsets (elements) and the byte
// offsets of each region inside the caller's reserve and scratch buffers.
struct PlanRegion {
    int which;           // 0: reserve, 1: scratch
    size_t offset, bytes;
};

struct Plan {
    std::vector<PlanRegion> regions;     // every region make_plan handed out
    int L, H, T, B, G, dtype, head, V, D;   // B: rows per time step = workers * per-worker batch
    int W = 1, Bw = 0;                       // simulated workers processed together, batch of each
    size_t es;                           // bytes per lp element
    std::vector<int> in_dim;             // I_l
    int F = 0;                           // units of the fully connected head layer (0: none)
    int64_t off_E = -1, off_wh = 0, off_bh = 0, off_Wfc = -1, off_bfc = -1, P = 0;
    size_t r_fc = 0;                     // reserve: relu(W_fc h + b_fc), lp [T*B, F]
    size_t s_fcd = 0, s_fcdT = 0, s_fcwT = 0;   // scratch: its gradient, the gradient transposed, W_fc^T
    int split_fc = 1;
    std::vector<int64_t> off_W, off_U, off_b;
    int head_rows = 0;                   // rows the head acts on (T*B or B)
    // reserve
    std::vector<size_t> r_gates, r_c, r_h, r_hblk;
    size_t r_xemb = 0, r_dzu = 0, r_xblk = 0, reserve_bytes = 0;
    bool blk = false;                    // whole-sequence GEMM operands are also kept in 64x64 blocks
    int h_ncb = 0, g_ncb = 0;            // column blocks of the blocked hidden sequence / dA
    size_t s_wblk = 0, s_dablk = 0;
    // scratch
    size_t s_ax = 0, s_cstate = 0, s_losspart = 0;
    size_t s_wT = 0, s_dA = 0, s_dAT = 0, s_xT = 0, s_dh[2] = {0, 0}, s_dhrec = 0, s_dcstate = 0, s_splitk = 0,
           s_colpart = 0, s_dE32 = 0, s_part = 0, s_upk = 0, s_apk[2] = {0, 0}, scratch_bytes = 0;
    // forward along anti-diagonals (cells of several layers per launch): per-layer operands and state
    bool wf = false, wb = false;   // wb: the backward pass too (costs one dA per layer, see make_plan)
    bool proj = false;             // large batches of narrow layers: the input projection runs inside the step kernels
    size_t s_pj_wpk = 0, s_pj_xseq = 0, s_pj_hseq[2] = {0, 0}, pj_slot_h = 0, pj_slot_x = 0;   // bytes
    bool fb = false;               // wb with each cell's products and gate arithmetic in one launch (narrow layers)
    // Wide layers (recurrent_tile.hip): the diagonal schedules with layer l running lag_c time steps behind the layer
    // it depends on, so that the projection that feeds it (forward: Ax of layer l from h of layer l - 1; backward: dh
    // of layer l from dA of layer l + 1) stays a whole-sequence GEMM over chunks of lag_c time steps
    bool lag = false;
    int lag_c = 32;
    std::vector<size_t> s_lag_ax, s_lag_dx, s_lag_wblk;
    // The chunk GEMMs on the packed-operand kernel (gemm_stream.hip): its A operand is the packed per-step copy the
    // recurrence writes anyway, kept for every time step instead of in two alternating buffers (s_lag_hseq: h_0 .. h_T
    // of the layers below the top, s_lag_daseq: dA_0 .. dA_{T-1} of the layers above the first); its B operand is W
    // packed like the recurrent matrix.  Projection: needs H % 256 == 0; data gradient: always.
    bool lag_sax = false, lag_sdx = false;
    std::vector<size_t> s_lag_hseq, s_lag_daseq;
    // lag_pk: nothing on the wide-layer path reads the 64x64-blocked copies of h_t and dA_t any more (the
    // weight-gradient GEMMs take the packed copies too): h_t is written in packed form only, into the region the
    // blocked sequence would occupy (same size; slot t = h_t), dA_t of the layers above the first into s_lag_daseq
    // only.  Layer 0 keeps its blocked dA: its dW (narrow input, split K) stays on the general kernel.  Needs the
    // diagonal backward form and T*B a multiple of 128 (the weight-gradient kernel's K granularity).
    bool lag_pk = false;
    // lag_x0: layer 0 as well (input width a multiple of 256): the input sequence is kept packed, in the region its
    // blocked copy would occupy, its projection runs on the packed-operand kernel and its dW on the weight-gradient
    // kernel with split K.  dA_0 then keeps a blocked copy only where the embedding's data gradient reads it.
    bool lag_x0 = false;
    std::vector<size_t> s_wb_dapk1; // second packed dA per layer (fb: a cell reads one step's while writing the next)
    std::vector<size_t> s_wf_upk, s_wf_wpk, s_wf_c, s_wf_hpk0, s_wf_hpk1;
    // backward along anti-diagonals: per-layer dA (row-major and blocked), packed U^T / W^T, packed dA_t,
    // the two sets of K-slice partials (dA U for the step before, dA W for the layer below), cell gradient
    std::vector<size_t> s_wb_dA, s_wb_dablk, s_wb_utpk, s_wb_wtpk, s_wb_dapk, s_wb_partU, s_wb_partW, s_wb_dc;
    std::vector<size_t> wT_off, uT_off;  // byte offsets inside the s_wT region
    // The row-major copy of dA is only kept where something reads it: with every consumer (dX, dW,
    // dU, the bias gradient) on the blocked copy it is left out.
    // wide layers whose dA has no blocked copy: every reader takes the packed per-step copies
    bool dA_packed_only(int l) const { return lag_pk && (l > 0 || (lag_x0 && V == 0)); }
    bool dA_rowmajor_needed(int l) const {
        if (!blk) return true;
        const int TB = T * B, I = in_dim[l];
        const bool dx = (l > 0 && !wb) || (l == 0 && V > 0);
        if (dx && !gemm_blocked_supported(dtype, TB, I)) return true;
        // dW takes the blocked kernel at any input width; dU too when there are several workers
        return W == 1 && !gemm_blocked_supported(dtype, G, H);
    }
    std::vector<int> split_w, split_u;
};

int make_plan(const lstm_config *c, Plan &p) {
    if (!c) {
        set_error("config is null");
        return LSTM_ERR_INVALID;
    }
    if (c->num_layers < 1 || c->hidden < 1 || c->seq_len < 1 || c->batch < 1) {
        set_error("config: num_layers, hidden, seq_len and batch must be >= 1");
        return LSTM_ERR_INVALID;
    }
    if (c->dtype < LSTM_DTYPE_FP32 || c->dtype > LSTM_DTYPE_BF16) {
        set_error("config: bad dtype %d", c->dtype);
        return LSTM_ERR_INVALID;
    }
    if (c->head < LSTM_HEAD_STEP_BCE || c->head > LSTM_HEAD_FC_HINGE) {
        set_error("config: bad head %d", c->head);
        return LSTM_ERR_INVALID;
    }
    if (c->head == LSTM_HEAD_FC_HINGE && (c->head_hidden < 1 || c->head_hidden > (1 << 20))) {
        set_error("config: head_hidden must be in [1, 2^20] with the fully connected head (got %d)", c->head_hidden);
        return LSTM_ERR_INVALID;
    }
    if (c->out_dim != 1) {
        set_error("config: out_dim must be 1 (got %d)", c->out_dim);
        return LSTM_ERR_UNSUPPORTED;
    }
    if (c->vocab < 0 || (c->vocab > 0 && c->embed_dim < 1) || (c->vocab == 0 && c->input_dim < 1)) {
        set_error("config: need input_dim >= 1, or vocab > 0 with embed_dim >= 1");
        return LSTM_ERR_INVALID;
    }
    const int64_t rows = (int64_t)c->seq_len * c->batch;
    if (rows > (int64_t)65535 * 64 || (int64_t)c->hidden * 4 > (1 << 24) || c->num_layers > 4096) {
        set_error("config: shape too large for this build (T*B=%lld, H=%d, L=%d)", (long long)rows, c->hidden, c->num_layers);
        return LSTM_ERR_UNSUPPORTED;
    }
    p.W = c->workers > 1 ? c->workers : 1;
    p.Bw = c->batch;
    if (p.W > 1) {
        if (c->dtype == LSTM_DTYPE_FP32 || c->batch % 64 != 0 || c->vocab > 0 || c->head == LSTM_HEAD_FC_HINGE || p.W > 4096 ||
            (int64_t)c->seq_len * c->batch * p.W > (int64_t)65535 * 64) {
            set_error("config: workers=%d needs a 16-bit type, batch %% 64 == 0, no embedding and a single-layer head", p.W);
            return LSTM_ERR_UNSUPPORTED;
        }
    }
    p.L = c->num_layers; p.H = c->hidden; p.T = c->seq_len; p.B = c->batch * p.W; p.G = 4 * c->hidden;
    p.dtype = c->dtype; p.head = c->head; p.V = c->vocab; p.D = c->vocab > 0 ? c->embed_dim : 0;
    p.F = c->head == LSTM_HEAD_FC_HINGE ? c->head_hidden : 0;
    p.es = dtype_size(c->dtype);
    const int I0 = c->vocab > 0 ? c->embed_dim : c->input_dim;
    p.in_dim.assign(p.L, p.H);
    p.in_dim[0] = I0;
    // ---- parameters
    int64_t off = 0;
    if (p.V > 0) { p.off_E = 0; off += (int64_t)p.V * p.D; }
    p.off_W.resize(p.L); p.off_U.resize(p.L); p.off_b.resize(p.L);
    for (int l = 0; l < p.L; ++l) {
        p.off_W[l] = off; off += (int64_t)p.G * p.in_dim[l];
        p.off_U[l] = off; off += (int64_t)p.G * p.H;
        p.off_b[l] = off; off += p.G;
    }
    if (p.F > 0) {
        p.off_Wfc = off; off += (int64_t)p.F * p.H;
        p.off_bfc = off; off += p.F;
    }
    p.off_wh = off; off += p.F > 0 ? p.F : p.H;
    p.off_bh = off; off += 1;
    p.P = off;
    p.head_rows = p.head == LSTM_HEAD_LAST_BCE ? p.B : p.T * p.B;
    // ---- reserve
    const size_t TB = (size_t)p.T * p.B;
    size_t r = 0, s = 0;
    // every region of the two workspaces is handed out here, 256-byte aligned, and remembered, so
    // that the plan can be checked for overlaps from the host (lstm_debug_plan_regions)
    p.regions.clear();
    auto take = [&](int which, size_t bytes) {
        size_t &cur = which == 0 ? r : s;
        const size_t off = cur;
        if (bytes > 0) p.regions.push_back(PlanRegion{which, off, bytes});
        cur += align_up(bytes);
        return off;
    };
    p.r_gates.resize(p.L); p.r_c.resize(p.L); p.r_h.resize(p.L);
    for (int l = 0; l < p.L; ++l) {
        p.r_gates[l] = take(0, TB * p.G * p.es);
        p.r_c[l] = take(0, (TB + p.B) * p.H * p.es);
        p.r_h[l] = take(0, (TB + p.B) * p.H * p.es);
    }
    p.r_xemb = r; if (p.V > 0) take(0, TB * p.D * p.es);
    p.r_dzu = take(0, (size_t)p.head_rows * 4);
    p.r_fc = r; if (p.F > 0) take(0, TB * p.F * p.es);
    // 64x64-blocked copies for the large-tile GEMMs: time slots must start on a block row
    p.blk = p.dtype != LSTM_DTYPE_FP32 && p.B % 64 == 0 && gemm_blocked_supported(p.dtype, (int)TB, p.G);
    // the blocked kernels address an operand with 32-bit element offsets: beyond that the row-major path runs
    const size_t blk_limit = (size_t)1 << 31;
    if (p.blk && (blocked_elems((int)TB, p.G) >= blk_limit || blocked_elems((int)(TB + p.B), p.H) >= blk_limit ||
                  blocked_elems((int)TB, p.in_dim[0]) >= blk_limit))
        p.blk = false;
    p.r_hblk.assign(p.L, 0);
    if (p.blk) {
        p.h_ncb = (p.H + 63) / 64;
        p.g_ncb = (p.G + 63) / 64;
        for (int l = 0; l < p.L; ++l) { p.r_hblk[l] = take(0, blocked_elems((int)(TB + p.B), p.H) * p.es); }
        p.r_xblk = take(0, blocked_elems((int)TB, p.in_dim[0]) * p.es);
    }
    p.reserve_bytes = r;
    // ---- scratch
    int max_in = 0;
    for (int l = 0; l < p.L; ++l) max_in = p.in_dim[l] > max_in ? p.in_dim[l] : max_in;
    const int max_dim = max_in > p.H ? max_in : p.H;
    p.s_ax = take(1, TB * p.G * 4);
    p.s_cstate = take(1, (size_t)p.B * p.H * 4);
    p.s_losspart = take(1, (size_t)head_loss_blocks(p.head_rows) * 4);
    p.s_wT = s;
    p.wT_off.resize(p.L); p.uT_off.resize(p.L);
    for (int l = 0; l < p.L; ++l) {
        p.wT_off[l] = take(1, (size_t)p.G * p.in_dim[l] * p.es) - p.s_wT;
        p.uT_off[l] = take(1, (size_t)p.G * p.H * p.es) - p.s_wT;
    }
    p.s_dA = take(1, TB * p.G * p.es);
    p.s_dAT = take(1, TB * p.G * p.es);
    p.s_xT = take(1, TB * max_dim * p.es);
    p.s_dh[0] = take(1, TB * max_dim * p.es);
    p.s_dh[1] = take(1, TB * max_dim * p.es);
    p.s_dhrec = take(1, (size_t)p.B * p.H * 4);
    p.s_dcstate = take(1, (size_t)p.B * p.H * 4);
    size_t splitk = 0;
    p.split_w.resize(p.L); p.split_u.resize(p.L);
    for (int l = 0; l < p.L; ++l) {
        p.split_w[l] = gemm_pick_splits(p.dtype, p.G, p.in_dim[l], (int)TB);
        p.split_u[l] = gemm_pick_splits(p.dtype, p.G, p.H, (int)TB);
        size_t a = p.split_w[l] > 1 ? (size_t)p.split_w[l] * p.G * p.in_dim[l] * 4 : 0;
        size_t b = p.split_u[l] > 1 ? (size_t)p.split_u[l] * p.G * p.H * 4 : 0;
        splitk = a > splitk ? a : splitk;
        splitk = b > splitk ? b : splitk;
    }
    if (p.F > 0) {
        p.split_fc = gemm_pick_splits(p.dtype, p.F, p.H, (int)TB);
        const size_t a = p.split_fc > 1 ? (size_t)p.split_fc * p.F * p.H * 4 : 0;
        splitk = a > splitk ? a : splitk;
    }
    p.s_splitk = take(1, splitk);
    if (p.F > 0) {
        p.s_fcd = take(1, TB * p.F * p.es);
        p.s_fcdT = take(1, TB * p.F * p.es);
        p.s_fcwT = take(1, (size_t)p.F * p.H * p.es);
    }
    const int colw = (p.G > p.H ? p.G : p.H) > p.F ? (p.G > p.H ? p.G : p.H) : p.F;
    {
        // partial column sums: the column-sum kernels' chunks, or the row groups of the one-launch backward recurrence
        size_t parts = (size_t)colsum_chunks((int)(TB / p.W)) * p.W;
        if (parts < (size_t)rows_backward_groups(p.B)) parts = (size_t)rows_backward_groups(p.B);
        p.s_colpart = take(1, parts * colw * 4);
    }
    p.s_dE32 = s; if (p.V > 0) take(1, (size_t)p.V * p.D * 4);
    if (p.dtype != LSTM_DTYPE_FP32) {
        // packed operands of the fused recurrent kernels
        const RecurrentDims rd = recurrent_dims(p.B, p.H);
        p.s_part = take(1, rd.partial_bytes);
        p.s_upk = take(1, (rd.utpk_elems > rd.upk_elems ? rd.utpk_elems : rd.upk_elems) * p.es);
        for (int k = 0; k < 2; ++k) { p.s_apk[k] = take(1, rd.dapk_elems * p.es); }
    }
    if (p.blk) {
        p.s_wblk = take(1, blocked_elems(p.G, max_dim) * p.es);
        p.s_dablk = take(1, blocked_elems((int)TB, p.G) * p.es);
    }
    if (p.dtype != LSTM_DTYPE_FP32) {
        const RecurrentDims rd = recurrent_dims(p.B, p.H);
        // The backward pass along the diagonals keeps every layer's dA (row-major and blocked) until
        // the weight-gradient GEMMs at the end, instead of one layer's at a time.  It is used while
        // that extra storage stays within a fixed budget; stacks deep enough to be bound by device
        // memory (the capacity experiment of Table 1) keep the layer-by-layer backward pass.
        auto diagonal_backward_fits = [&]() {
            constexpr size_t kDiagonalBackwardBudget = (size_t)8 << 30;
            const bool wb_was = p.wb;
            p.wb = true;                                       // dA_rowmajor_needed() asks as if the form were on
            size_t extra = 0;
            for (int l = 0; l < p.L; ++l)
                extra += (p.dA_rowmajor_needed(l) ? align_up(TB * p.G * p.es) : 0) +
                         (p.blk ? align_up(blocked_elems((int)TB, p.G) * p.es) : 0) + 2 * align_up(rd.utpk_elems * p.es) +
                         2 * align_up(rd.dapk_elems * p.es) + 2 * align_up(rd.partial_bytes) + align_up((size_t)p.B * p.H * 4) +
                         (p.lag ? align_up((size_t)p.T * rd.dapk_elems * p.es) : 0);
            p.wb = wb_was;
            return extra <= kDiagonalBackwardBudget;
        };
        // Stacks of narrow layers: a time step of one layer is a handful of workgroups, so the
        // forward pass runs along anti-diagonals (all layers' ready cells in one launch).
        p.wf = p.L >= 2 && rd.n_mt * rd.n_hb <= 128;
        // wide layers: a cell is hundreds of workgroups and bound by operand traffic; the tile kernels with the
        // layers' cells sharing launches (any depth: a single layer simply has one cell per launch)
        p.lag = !p.wf && p.W == 1 && p.blk && p.H >= 1024 && p.B >= 192 && tile_kernels_supported(p.dtype, p.B, p.H);
        if (p.lag) {
            p.wf = true;
            // 32 steps: the chunk GEMMs (32 * B rows) are large enough to run near the whole-sequence rate, and the
            // ramps at both ends of the schedule (launches with fewer cells than layers) stay short.  Measured on
            // the 3 x 2048-unit model, T = 128, B = 256: 16 steps 24.9 ms per training step, 24: 23.9, 32: 23.7,
            // 48: 24.2, 64: 24.7, 128 (no overlap between layers): 26.0
            p.lag_c = p.T < 32 ? p.T : 32;
            p.s_lag_ax.assign(p.L, 0); p.s_lag_dx.assign(p.L, 0); p.s_lag_wblk.assign(p.L, 0);
            p.s_lag_hseq.assign(p.L, 0); p.s_lag_daseq.assign(p.L, 0);
            p.lag_sax = p.H % 256 == 0;
            p.lag_sdx = true;
            p.lag_pk = p.lag_sax && TB % 128 == 0 && gemm_blocked_supported(p.dtype, p.G, p.H) &&
                       (size_t)(p.T + 1) * rd.hpk_elems <= blocked_elems((int)(TB + p.B), p.H) && diagonal_backward_fits();
            // (the kernel that takes packed weight-gradient operands has no split-K form)
            for (int l = 0; l < p.L; ++l) p.lag_pk = p.lag_pk && p.split_u[l] == 1 && (l == 0 || p.split_w[l] == 1);
            p.lag_x0 = p.lag_pk && p.in_dim[0] % 256 == 0 && TB % (128 * (size_t)p.split_w[0]) == 0;
            for (int l = 1; l < p.L; ++l) {
                p.s_lag_ax[l] = take(1, (size_t)p.lag_c * p.B * p.G * p.es);
                p.s_lag_dx[l - 1] = take(1, (size_t)p.lag_c * p.B * p.H * p.es);
                if (!p.lag_sax) p.s_lag_wblk[l] = take(1, blocked_elems(p.G, p.H) * p.es);
                if (p.lag_sax && !p.lag_pk) p.s_lag_hseq[l - 1] = take(1, (size_t)(p.T + 1) * rd.hpk_elems * p.es);
            }
        }
        if (p.wf) {
            p.s_wf_upk.resize(p.L); p.s_wf_wpk.assign(p.L, 0); p.s_wf_c.resize(p.L); p.s_wf_hpk0.resize(p.L); p.s_wf_hpk1.resize(p.L);
            for (int l = 0; l < p.L; ++l) {
                p.s_wf_upk[l] = take(1, rd.upk_elems * p.es);
                if (l > 0 && (!p.lag || p.lag_sax)) { p.s_wf_wpk[l] = take(1, rd.upk_elems * p.es); }
                if (l == 0 && p.lag_x0) { p.s_wf_wpk[0] = take(1, (size_t)p.G * p.in_dim[0] * p.es); }
                p.s_wf_hpk0[l] = take(1, rd.hpk_elems * p.es);
                p.s_wf_hpk1[l] = take(1, rd.hpk_elems * p.es);
                p.s_wf_c[l] = take(1, (size_t)p.B * p.H * 4);
            }
        }
        // Thousands of rows per step on narrow layers: a whole-sequence input projection is bound by writing and
        // re-reading its [T*B, 4H] result, so the step kernels project their own input (W packed like U, the
        // layer's input sequence packed step by step; a layer's packed h_t sequence is the next layer's input).
        p.proj = !p.wf && recurrent_wide_shape(p.B, p.H) && !fused_backward_supported(p.dtype, p.B, p.H);   // beyond the narrow-layer kernels' range
        if (p.proj) {
            int max_in = 1;
            for (int l = 0; l < p.L; ++l) max_in = p.in_dim[l] > max_in ? p.in_dim[l] : max_in;
            const size_t b_chunk = rd.upk_elems / ((size_t)rd.n_hb * rd.nkc), a_chunk = rd.hpk_elems / ((size_t)rd.n_mt * rd.nkc);
            p.s_pj_wpk = take(1, (size_t)rd.n_hb * ((max_in + 63) / 64) * b_chunk * p.es);
            p.pj_slot_h = align_up(rd.hpk_elems * p.es);
            p.pj_slot_x = align_up((size_t)rd.n_mt * ((p.in_dim[0] + 63) / 64) * a_chunk * p.es);
            p.s_pj_xseq = take(1, (size_t)p.T * p.pj_slot_x);
            for (int k = 0; k < 2; ++k) p.s_pj_hseq[k] = take(1, (size_t)(p.T + 1) * p.pj_slot_h);
        }
        // Narrow layers of any depth: each BPTT cell in one launch instead of two.
        const bool fb_ok = fused_backward_supported(p.dtype, p.B, p.H);
        if (p.wf || fb_ok) p.wb = diagonal_backward_fits();
        p.fb = p.wb && fb_ok;
        if (p.wb) {
            p.s_wb_dA.resize(p.L); p.s_wb_dablk.assign(p.L, 0); p.s_wb_utpk.resize(p.L); p.s_wb_wtpk.assign(p.L, 0);
            p.s_wb_dapk.resize(p.L); p.s_wb_dapk1.assign(p.L, 0); p.s_wb_partU.resize(p.L); p.s_wb_partW.assign(p.L, 0);
            p.s_wb_dc.resize(p.L);
            for (int l = 0; l < p.L; ++l) {
                p.s_wb_dA[l] = s; if (p.dA_rowmajor_needed(l)) take(1, TB * p.G * p.es);
                if (p.blk && !p.dA_packed_only(l)) { p.s_wb_dablk[l] = take(1, blocked_elems((int)TB, p.G) * p.es); }
                p.s_wb_utpk[l] = take(1, rd.utpk_elems * p.es);
                if (l > 0 && (!p.lag || p.lag_sdx)) { p.s_wb_wtpk[l] = take(1, rd.utpk_elems * p.es); }
                if (p.lag && p.lag_sdx && (l > 0 || p.lag_pk)) { p.s_lag_daseq[l] = take(1, (size_t)p.T * rd.dapk_elems * p.es); }
                p.s_wb_dapk[l] = take(1, rd.dapk_elems * p.es);
                if (p.fb) { p.s_wb_dapk1[l] = take(1, rd.dapk_elems * p.es); }
                p.s_wb_partU[l] = s; if (!p.fb) take(1, rd.partial_bytes);
                if (l > 0 && !p.fb && !p.lag) { p.s_wb_partW[l] = take(1, rd.partial_bytes); }
                p.s_wb_dc[l] = take(1, (size_t)p.B * p.H * 4);
            }
        }
    }
    p.scratch_bytes = s;
    if (p.W > 1 && !p.blk) {
        set_error("config: workers=%d needs shapes the blocked GEMM path handles (T*W*B >= 192, 4H >= 192, T*W*B*4H < 2^31)", p.W);
        return LSTM_ERR_UNSUPPORTED;
    }
    return LSTM_OK;
}

inline char *at(void *base, size_t off) { return reinterpret_cast<char *>(base) + off; }
inline const char *at(const void *base, size_t off) { return reinterpret_cast<const char *>(base) + off; }

// The packing jobs and zero fills a pass starts with, collected and sent as one launch (16-bit types;
// the fp32 mode has no packed operands and keeps its plain fills).
struct SetupBatch {
    std::vector<SetupJob> jobs;
    void pack_u_forward(const void *U, void *dst) { jobs.push_back(SetupJob{SETUP_PACK_U_FORWARD, U, dst, 0, 0, 0}); }
    void pack_u_backward(const void *U, void *dst) { jobs.push_back(SetupJob{SETUP_PACK_U_BACKWARD, U, dst, 0, 0, 0}); }
    void pack_rows(const void *h, void *dst) { jobs.push_back(SetupJob{SETUP_PACK_ROWS, h, dst, 0, 0, 0}); }
    void zero(void *dst, int64_t n_words) { if (n_words > 0) jobs.push_back(SetupJob{SETUP_ZERO, nullptr, dst, n_words, 0, 0}); }
    // padding columns of a 64x64-blocked [rows, cols] tensor (the kernels that fill it write valid columns only)
    void zero_pad(void *dst, int64_t rows, int cols) {
        if (cols % 64 != 0 && rows > 0) jobs.push_back(SetupJob{SETUP_ZERO_PAD, nullptr, dst, (rows + 63) / 64, (cols + 63) / 64, cols});
    }
    int flush(int dtype, int B, int H, hipStream_t s) {
        if (jobs.empty()) return LSTM_OK;
        const int rc = setup_jobs(dtype, jobs.data(), (int)jobs.size(), B, H, s);
        jobs.clear();
        return rc;
    }
};

int check_ptr(const void *p, const char *name, bool required = true) {
    if (!p) {
        if (!required) return LSTM_OK;
        set_error("%s is null", name);
        return LSTM_ERR_INVALID;
    }
    if ((uintptr_t)p % 16 != 0) {
        set_error("%s is not 16-byte aligned", name);
        return LSTM_ERR_INVALID;
    }
    return LSTM_OK;
}

}  // namespace
}  // namespace lstm

using namespace lstm;

extern "C" int lstm_abi_version(void) { return LSTM_ABI_VERSION; }

extern "C" const char *lstm_last_error(void) { return g_err; }

extern "C" int lstm_param_count(const lstm_config *cfg, int64_t *n_params) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    if (!n_params) {
        set_error("n_params is null");
        return LSTM_ERR_INVALID;
    }
    *n_params = p.P;
    return LSTM_OK;
}

extern "C" int lstm_param_offset(const lstm_config *cfg, int32_t kind, int32_t layer, int64_t *offset, int64_t *count) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    if (!offset || !count) {
        set_error("offset/count is null");
        return LSTM_ERR_INVALID;
    }
    const bool per_layer = kind == LSTM_P_W || kind == LSTM_P_U || kind == LSTM_P_B;
    if (per_layer && (layer < 0 || layer >= p.L)) {
        set_error("layer %d out of range", layer);
        return LSTM_ERR_INVALID;
    }
    switch (kind) {
        case LSTM_P_EMBED:
            if (p.V == 0) {
                set_error("config has no embedding");
                return LSTM_ERR_INVALID;
            }
            *offset = p.off_E; *count = (int64_t)p.V * p.D; break;
        case LSTM_P_W: *offset = p.off_W[layer]; *count = (int64_t)p.G * p.in_dim[layer]; break;
        case LSTM_P_U: *offset = p.off_U[layer]; *count = (int64_t)p.G * p.H; break;
        case LSTM_P_B: *offset = p.off_b[layer]; *count = p.G; break;
        case LSTM_P_HEAD_W: *offset = p.off_wh; *count = p.F > 0 ? p.F : p.H; break;
        case LSTM_P_FC_W:
        case LSTM_P_FC_B:
            if (p.F == 0) {
                set_error("config has no fully connected head layer");
                return LSTM_ERR_INVALID;
            }
            *offset = kind == LSTM_P_FC_W ? p.off_Wfc : p.off_bfc;
            *count = kind == LSTM_P_FC_W ? (int64_t)p.F * p.H : p.F;
            break;
        case LSTM_P_HEAD_B: *offset = p.off_bh; *count = 1; break;
        default:
            set_error("unknown tensor kind %d", kind);
            return LSTM_ERR_INVALID;
    }
    return LSTM_OK;
}

extern "C" int lstm_workspace_bytes(const lstm_config *cfg, size_t *reserve_bytes, size_t *scratch_bytes) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    if (!reserve_bytes || !scratch_bytes) {
        set_error("reserve_bytes/scratch_bytes is null");
        return LSTM_ERR_INVALID;
    }
    *reserve_bytes = p.reserve_bytes;
    *scratch_bytes = p.scratch_bytes;
    return LSTM_OK;
}

// the caller's buffers against the plan: an undersized workspace is refused before anything is enqueued
static int check_workspace(const Plan &p, size_t reserve_bytes, size_t scratch_bytes) {
    if (reserve_bytes < p.reserve_bytes || scratch_bytes < p.scratch_bytes) {
        set_error("workspace too small for this config: reserve %zu of %zu bytes, scratch %zu of %zu bytes (see lstm_workspace_bytes)",
                  reserve_bytes, p.reserve_bytes, scratch_bytes, p.scratch_bytes);
        return LSTM_ERR_WORKSPACE;
    }
    return LSTM_OK;
}

extern "C" int lstm_forward(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                            const void *h0, const float *c0, void *reserve, size_t reserve_bytes, void *scratch,
                            size_t scratch_bytes, float *loss, void *hT, float *cT, void *stream) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    LSTM_TRY(check_workspace(p, reserve_bytes, scratch_bytes));
    LSTM_TRY(check_ptr(params_lp, "params_lp"));
    LSTM_TRY(check_ptr(x, "x"));
    LSTM_TRY(check_ptr(targets, "targets"));
    LSTM_TRY(check_ptr(reserve, "reserve"));
    LSTM_TRY(check_ptr(scratch, "scratch"));
    LSTM_TRY(check_ptr(h0, "h0", false));
    LSTM_TRY(check_ptr(c0, "c0", false));
    LSTM_TRY(check_ptr(hT, "hT", false));
    LSTM_TRY(check_ptr(cT, "cT", false));
    if (!loss) {
        set_error("loss is null");
        return LSTM_ERR_INVALID;
    }
    hipStream_t s = (hipStream_t)stream;
    const size_t es = p.es;
    const int TB = p.T * p.B;
    const char *par = reinterpret_cast<const char *>(params_lp);
    const int64_t BH = (int64_t)p.B * p.H;

    const void *layer_in = x;
    if (p.V > 0) {
        void *xe = at(reserve, p.r_xemb);
        LSTM_TRY(embed_gather(p.dtype, (const int32_t *)x, par + p.off_E * es, xe, TB, p.V, p.D, s));
        layer_in = xe;
    }
    // input projection of a whole layer: fp32 in the fp32 baseline mode (the recurrent GEMM
    // accumulates into it), otherwise stored in the 16-bit type like every other activation
    char *ax = at(scratch, p.s_ax);
    const bool fused = p.dtype != LSTM_DTYPE_FP32;
    const size_t axs = fused ? es : 4;
    // wide layers: packed h_0 .. h_T of layer l, one slot per step (in place of the blocked sequence when nothing reads that)
    auto lag_hseq = [&](int l) { return p.lag_pk ? at(reserve, p.r_hblk[l]) : at(scratch, p.s_lag_hseq[l]); };
    SetupBatch setup;
    for (int l = 0; l < p.L; ++l) {
        const void *W = par + p.off_W[l] * es, *U = par + p.off_U[l] * es, *b = par + p.off_b[l] * es;
        char *gates = at(reserve, p.r_gates[l]);
        char *cs = at(reserve, p.r_c[l]);
        char *hs = at(reserve, p.r_h[l]);
        float *c_state = (float *)at(scratch, p.wf ? p.s_wf_c[l] : p.s_cstate);
        // input projection of the whole sequence: Ax = X W^T + b  (along the anti-diagonals only
        // layer 0 has its input ahead of time; the layers above project inside their step kernels)
        if (l == 0 && p.lag_x0) {
            // the packed-operand kernel: x packed step by step like the h_t sequences, W like the recurrent matrix
            const int I = p.in_dim[0];
            LSTM_TRY(pack_w_forward(p.dtype, W, at(scratch, p.s_wf_wpk[0]), p.H, I, s));
            LSTM_TRY(pack_rows_seq(p.dtype, layer_in, at(reserve, p.r_xblk), p.T, p.B, I, (int64_t)p.B * I, s));
            StreamGemmArgs g{};
            g.A = at(reserve, p.r_xblk); g.a_step_stride = (int64_t)p.B * I; g.rows_per_step = p.B;
            g.B = at(scratch, p.s_wf_wpk[0]); g.gate_h = p.H;
            g.C = ax; g.bias = b; g.ldc = p.G;
            g.M = (int)TB; g.N = p.G; g.K = I;
            g.kclass = KC_GEMM_BATCHED;
            LSTM_TRY(gemm_stream(p.dtype, g, s));
        } else if (p.lag && l > 0 && !p.lag_sax) {
            // projected chunk by chunk between the step launches below: W in 64x64 blocks once
            LSTM_TRY(pack_blocked(p.dtype, W, p.in_dim[l], p.G, p.in_dim[l], at(scratch, p.s_lag_wblk[l]), s));
        } else if (p.wf && l > 0) {
            // (wide layers: the B operand of the chunked projection on the packed-operand kernel)
            setup.pack_u_forward(W, at(scratch, p.s_wf_wpk[l]));
        } else if (p.proj) {
            // the step kernels project their own input: W packed like U; layer 0's input sequence packed step by
            // step (the layers above read the packed h_t sequence of the layer below)
            LSTM_TRY(pack_w_forward(p.dtype, W, at(scratch, p.s_pj_wpk), p.H, p.in_dim[l], s));
            if (l == 0) {
                if (p.blk)   // the weight-gradient GEMM of layer 0 reads the blocked copy
                    LSTM_TRY(pack_blocked(p.dtype, layer_in, p.in_dim[0], TB, p.in_dim[0], at(reserve, p.r_xblk), s));
                LSTM_TRY(pack_rows_seq(p.dtype, layer_in, at(scratch, p.s_pj_xseq), p.T, p.B, p.in_dim[0], (int64_t)(p.pj_slot_x / es), s));
            }
        } else if (p.blk) {
            // operands in 64x64 blocks: layer 0 packs the input once, upper layers read the blocked
            // hidden sequence the step kernels of the layer below wrote
            char *wblk = at(scratch, p.s_wblk);
            LSTM_TRY(pack_blocked(p.dtype, W, p.in_dim[l], p.G, p.in_dim[l], wblk, s));
            BlockedGemmArgs g{};
            if (l == 0) {
                LSTM_TRY(pack_blocked(p.dtype, layer_in, p.in_dim[0], TB, p.in_dim[0], at(reserve, p.r_xblk), s));
                g.A = BlockedOperand{at(reserve, p.r_xblk), (p.in_dim[0] + 63) / 64, 0};
            } else {
                g.A = BlockedOperand{at(reserve, p.r_hblk[l - 1]) + (size_t)(p.B / 64) * p.h_ncb * 4096 * es, p.h_ncb, 0};
            }
            g.B = BlockedOperand{wblk, (p.in_dim[l] + 63) / 64, 0};
            g.C = ax; g.bias = b; g.ldc = p.G; g.out_lp = 1;
            g.M = TB; g.N = p.G; g.K = p.in_dim[l];
            g.kclass = KC_GEMM_BATCHED;
            LSTM_TRY(gemm_blocked(p.dtype, g, s));
        } else {
            GemmArgs g{};
            g.A = layer_in; g.B = W; g.C = ax; g.bias = b;
            g.M = TB; g.N = p.G; g.K = p.in_dim[l];
            g.lda = p.in_dim[l]; g.ldb = p.in_dim[l]; g.ldc = p.G;
            g.out_lp = fused ? 1 : 0;
            g.kclass = KC_GEMM_BATCHED;
            LSTM_TRY(gemm_nt(p.dtype, g, s));
        }
        LSTM_TRY(init_state(p.dtype, h0 ? at(h0, (size_t)l * BH * es) : nullptr, c0 ? c0 + l * BH : nullptr, hs, cs,
                            c_state, BH, s));
        char *upk = at(scratch, p.wf ? p.s_wf_upk[l] : p.s_upk);
        char *hpk[2] = {at(scratch, p.wf ? p.s_wf_hpk0[l] : p.s_apk[0]), at(scratch, p.wf ? p.s_wf_hpk1[l] : p.s_apk[1])};
        if (p.lag && p.lag_sax && (l < p.L - 1 || p.lag_pk)) hpk[0] = lag_hseq(l);   // slot 0 of the kept sequence
        char *hseq = p.proj ? at(scratch, p.s_pj_hseq[l & 1]) : nullptr;    // packed h_0 .. h_T of this layer, one slot per step
        if (fused) {
            // recurrent weights and the initial hidden state in packed tile order; the second
            // packed-h buffer only needs its zero padding (the per-step slots of the projection mode get
            // theirs from the step kernels)
            setup.pack_u_forward(U, upk);
            setup.pack_rows(h0 ? at(h0, (size_t)l * BH * es) : nullptr, p.proj ? hseq : hpk[0]);
            if (!p.proj) setup.pack_rows(nullptr, hpk[1]);
        }
        char *hblk = (p.blk && !p.lag_pk) ? at(reserve, p.r_hblk[l]) : nullptr;
        const size_t slot = (size_t)(p.B / 64) * p.h_ncb * 4096 * es;      // bytes of one time slot of the blocked sequence
        if (hblk) {
            // zero padding columns (H not a multiple of 64) once, then slot 0 = initial hidden state
            setup.zero_pad(hblk, (int64_t)TB + p.B, p.H);
            if (!h0) setup.zero(hblk, (int64_t)(slot / 4));
            if (h0) {
                LSTM_TRY(setup.flush(p.dtype, p.B, p.H, s));     // the padding is cleared before slot 0 is written
                LSTM_TRY(pack_blocked(p.dtype, at(h0, (size_t)l * BH * es), p.H, p.B, p.H, hblk, s));
            }
        }
        if (p.wf) continue;                                   // the time steps follow below, diagonal by diagonal
        LSTM_TRY(setup.flush(p.dtype, p.B, p.H, s));
        const bool rows = fused && p.proj && rows_forward_supported(p.dtype, p.B, p.H, p.in_dim[l]);
        if (rows) {
            // every workgroup walks its 32 rows through all T steps: one launch for the layer
            RowsForward r{};
            r.hseq = hseq; r.slot_h = (int64_t)(p.pj_slot_h / es);
            r.xseq = l == 0 ? at(scratch, p.s_pj_xseq) : at(scratch, p.s_pj_hseq[(l - 1) & 1]) + p.pj_slot_h;
            r.slot_x = (int64_t)((l == 0 ? p.pj_slot_x : p.pj_slot_h) / es);
            r.Upk = upk; r.Wpk = at(scratch, p.s_pj_wpk); r.bias = b;
            r.c_state = c_state; r.gates = gates; r.c_out = cs + (size_t)BH * es; r.h_out = hs + (size_t)BH * es;
            r.h_blk = hblk ? hblk + slot : nullptr; r.slot_blk = (int64_t)(slot / es); r.blk_ncb = p.h_ncb;
            // row-major h_t: the head reads the top layer's, and this layer's dU product reads it unless it takes the
            // blocked copy (same condition as in lstm_backward); packed h_t: the layer above's input
            const bool u_blk = p.blk && (p.W > 1 || gemm_blocked_supported(p.dtype, p.G, p.H));
            r.all_h_out = (l == p.L - 1 || !u_blk) ? 1 : 0;
            r.write_hpk = l + 1 < p.L ? 1 : 0;
            LSTM_TRY(rows_forward(p.dtype, r, p.in_dim[l], p.T, p.B, p.H, s));
        }
        for (int t = rows ? p.T : 0; t < p.T; ++t) {
            char *a_t = ax + (size_t)t * p.B * p.G * axs;
            if (fused && p.proj) {
                const char *xin = l == 0 ? at(scratch, p.s_pj_xseq) + (size_t)t * p.pj_slot_x
                                         : at(scratch, p.s_pj_hseq[(l - 1) & 1]) + (size_t)(t + 1) * p.pj_slot_h;
                LSTM_TRY(step_forward_proj(p.dtype, hseq + (size_t)t * p.pj_slot_h, upk, xin, at(scratch, p.s_pj_wpk), b, p.in_dim[l],
                                           c_state, gates + (size_t)t * p.B * p.G * es, cs + (size_t)(t + 1) * BH * es,
                                           hs + (size_t)(t + 1) * BH * es, hseq + (size_t)(t + 1) * p.pj_slot_h,
                                           hblk ? hblk + (size_t)(t + 1) * slot : nullptr, p.h_ncb, p.B, p.H, s));
                continue;
            }
            if (fused) {
                // recurrent projection, gates, cell and hidden update in one launch
                LSTM_TRY(step_forward_fused(p.dtype, hpk[t & 1], upk, a_t, c_state, gates + (size_t)t * p.B * p.G * es,
                                            cs + (size_t)(t + 1) * BH * es, hs + (size_t)(t + 1) * BH * es,
                                            hpk[(t + 1) & 1], hblk ? hblk + (size_t)(t + 1) * slot : nullptr, p.h_ncb, p.B,
                                            p.H, s));
                continue;
            }
            // fp32 baseline mode: recurrent projection added in place (A_t += h_{t-1} U^T), then the gates
            GemmArgs r{};
            r.A = hs + (size_t)t * BH * es; r.B = U; r.C = a_t;   // fp32 here
            r.M = p.B; r.N = p.G; r.K = p.H;
            r.lda = p.H; r.ldb = p.H; r.ldc = p.G;
            r.accumulate = 1;
            r.kclass = KC_GEMM_STEP;
            LSTM_TRY(gemm_nt(p.dtype, r, s));
            LSTM_TRY(gates_forward(p.dtype, (const float *)a_t, c_state, gates + (size_t)t * p.B * p.G * es,
                                   cs + (size_t)(t + 1) * BH * es, hs + (size_t)(t + 1) * BH * es, p.B, p.H, s));
        }
        LSTM_TRY(copy_state(p.dtype, hs + (size_t)p.T * BH * es, c_state, hT ? at(hT, (size_t)l * BH * es) : nullptr,
                            cT ? cT + l * BH : nullptr, BH, s));
        layer_in = hs + (size_t)BH * es;   // h_1..h_T feed the next layer
    }
    if (p.wf) {
        LSTM_TRY(setup.flush(p.dtype, p.B, p.H, s));              // every layer's packing in one launch
        // cell (l, t) needs (l, t-1) and (l-1, t): all cells with l + t = d are independent
        const int max_cells = wave_forward_max_cells();
        const size_t slot = p.blk ? (size_t)(p.B / 64) * p.h_ncb * 4096 * es : 0;
        std::vector<WaveCell> cells;
        // wide layers: layer l runs lag_c steps behind layer l - 1, and takes its input projection from a
        // whole-sequence GEMM over the lag_c steps the layer below has just finished
        const int lag = p.lag ? p.lag_c : 1, max_launch = p.lag ? tile_max_cells() : max_cells;
        for (int d = 0; d < p.T + (p.L - 1) * lag; ++d) {
            cells.clear();
            for (int l = 1; p.lag && l < p.L; ++l) {
                const int t0 = d - l * lag;
                if (t0 < 0 || t0 >= p.T || t0 % lag != 0) continue;
                const int nt = p.T - t0 < lag ? p.T - t0 : lag;
                if (p.lag_sax) {
                    const RecurrentDims rd = recurrent_dims(p.B, p.H);
                    StreamGemmArgs g{};
                    g.A = lag_hseq(l - 1) + (size_t)(t0 + 1) * rd.hpk_elems * es;
                    g.a_step_stride = (int64_t)rd.hpk_elems; g.rows_per_step = p.B;
                    g.B = at(scratch, p.s_wf_wpk[l]); g.gate_h = p.H;
                    g.C = at(scratch, p.s_lag_ax[l]); g.bias = par + p.off_b[l] * es; g.ldc = p.G;
                    g.M = nt * p.B; g.N = p.G; g.K = p.in_dim[l];
                    g.kclass = KC_GEMM_BATCHED;
                    LSTM_TRY(gemm_stream(p.dtype, g, s));
                    continue;
                }
                BlockedGemmArgs g{};
                g.A = BlockedOperand{at(reserve, p.r_hblk[l - 1]) + (size_t)(t0 + 1) * slot, p.h_ncb, 0};
                g.B = BlockedOperand{at(scratch, p.s_lag_wblk[l]), (p.in_dim[l] + 63) / 64, 0};
                g.C = at(scratch, p.s_lag_ax[l]); g.bias = par + p.off_b[l] * es; g.ldc = p.G; g.out_lp = 1;
                g.M = nt * p.B; g.N = p.G; g.K = p.in_dim[l];
                g.kclass = KC_GEMM_BATCHED;
                LSTM_TRY(gemm_blocked(p.dtype, g, s));
            }
            for (int l = 0; l < p.L; ++l) {
                const int t = d - l * lag;
                if (t < 0 || t >= p.T) continue;
                char *hpk[2] = {at(scratch, p.s_wf_hpk0[l]), at(scratch, p.s_wf_hpk1[l])};
                WaveCell c{};
                c.hpk_prev = hpk[t & 1]; c.hpk_next = hpk[(t + 1) & 1];
                if (p.lag && p.lag_sax && (l < p.L - 1 || p.lag_pk)) {
                    const size_t hpk_bytes = recurrent_dims(p.B, p.H).hpk_elems * es;
                    c.hpk_prev = lag_hseq(l) + (size_t)t * hpk_bytes;
                    c.hpk_next = lag_hseq(l) + (size_t)(t + 1) * hpk_bytes;
                }
                c.Upk = at(scratch, p.s_wf_upk[l]);
                if (l == 0) {
                    c.Ax = ax + (size_t)t * p.B * p.G * axs;
                } else if (p.lag) {
                    c.Ax = at(scratch, p.s_lag_ax[l]) + (size_t)(t % lag) * p.B * p.G * es;
                } else {
                    // packed h_t of the layer below: written one launch ago into its buffer (t + 1) % 2
                    c.xpk = at(scratch, ((t + 1) & 1) ? p.s_wf_hpk1[l - 1] : p.s_wf_hpk0[l - 1]);
                    c.Wpk = at(scratch, p.s_wf_wpk[l]);
                    c.bias = par + p.off_b[l] * es;
                }
                c.c_state = (float *)at(scratch, p.s_wf_c[l]);
                c.gates = at(reserve, p.r_gates[l]) + (size_t)t * p.B * p.G * es;
                c.c_out = at(reserve, p.r_c[l]) + (size_t)(t + 1) * BH * es;
                c.h_out = at(reserve, p.r_h[l]) + (size_t)(t + 1) * BH * es;
                c.h_blk = (p.blk && !p.lag_pk) ? at(reserve, p.r_hblk[l]) + (size_t)(t + 1) * slot : nullptr;
                // row-major h_t: the head reads the top layer's and the final state is copied out of the last step's;
                // everything else on the wide-layer path reads the packed or the blocked copy
                if (p.lag && l < p.L - 1 && t < p.T - 1 && gemm_blocked_supported(p.dtype, p.G, p.H)) c.h_out = nullptr;
                cells.push_back(c);
                if ((int)cells.size() == max_launch) {
                    LSTM_TRY((p.lag ? step_forward_tile : step_forward_wave)(p.dtype, cells.data(), (int)cells.size(), p.h_ncb, p.B, p.H, s));
                    cells.clear();
                }
            }
            if (!cells.empty())
                LSTM_TRY((p.lag ? step_forward_tile : step_forward_wave)(p.dtype, cells.data(), (int)cells.size(), p.h_ncb, p.B, p.H, s));
        }
        for (int l = 0; l < p.L; ++l)
            LSTM_TRY(copy_state(p.dtype, at(reserve, p.r_h[l]) + (size_t)p.T * BH * es, (const float *)at(scratch, p.s_wf_c[l]),
                                hT ? at(hT, (size_t)l * BH * es) : nullptr, cT ? cT + l * BH : nullptr, BH, s));
    }
    // head + loss on the top layer's outputs
    const char *top = at(reserve, p.r_h[p.L - 1]) + (size_t)BH * es;
    if (p.head == LSTM_HEAD_LAST_BCE) top += (size_t)(p.T - 1) * BH * es;
    int head_width = p.H;
    if (p.F > 0) {
        // Fig. 2: fully connected ReLU layer on every temporal slice, a = relu(h W_fc^T + b_fc)
        char *act = at(reserve, p.r_fc);
        GemmArgs g{};
        g.A = top; g.B = par + p.off_Wfc * es; g.C = act; g.bias = par + p.off_bfc * es;
        g.M = TB; g.N = p.F; g.K = p.H;
        g.lda = p.H; g.ldb = p.H; g.ldc = p.F;
        g.out_lp = 1; g.kclass = KC_GEMM_BATCHED;
        LSTM_TRY(gemm_nt(p.dtype, g, s));
        LSTM_TRY(relu_inplace(p.dtype, act, (int64_t)TB * p.F, s));
        top = act;
        head_width = p.F;
    }
    LSTM_TRY(head_forward(p.dtype, p.head, top, par + p.off_wh * es, par + p.off_bh * es, targets, p.head_rows, head_width,
                          p.head_rows / p.W, (float *)at(reserve, p.r_dzu), (float *)at(scratch, p.s_losspart), loss, s, p.W,
                          p.Bw));
    return LSTM_OK;
}

extern "C" int lstm_backward(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                             const void *reserve, size_t reserve_bytes, void *scratch, size_t scratch_bytes,
                             const float *loss_scale, void *grads_lp, void *stream) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    LSTM_TRY(check_workspace(p, reserve_bytes, scratch_bytes));
    LSTM_TRY(check_ptr(params_lp, "params_lp"));
    LSTM_TRY(check_ptr(x, "x"));
    LSTM_TRY(check_ptr(reserve, "reserve"));
    LSTM_TRY(check_ptr(scratch, "scratch"));
    // one worker's row of an [N,P] gradient matrix: only element alignment can be asked for
    if (!grads_lp || (uintptr_t)grads_lp % p.es != 0) {
        set_error("grads_lp is null or not aligned to its element size");
        return LSTM_ERR_INVALID;
    }
    if (!loss_scale) {
        set_error("loss_scale is null");
        return LSTM_ERR_INVALID;
    }
    (void)targets;  // the head's derivative was saved by lstm_forward
    hipStream_t s = (hipStream_t)stream;
    const size_t es = p.es;
    const int TB = p.T * p.B;
    const int64_t BH = (int64_t)p.B * p.H;
    const char *par = reinterpret_cast<const char *>(params_lp);
    char *grd = reinterpret_cast<char *>(grads_lp);
    const float *dzu = (const float *)at(reserve, p.r_dzu);
    float *colpart = (float *)at(scratch, p.s_colpart);
    float *splitk = (float *)at(scratch, p.s_splitk);
    char *wT = at(scratch, p.s_wT);

    // transposed copies of the weights the data-gradient GEMMs contract over
    for (int l = 0; l < p.L; ++l) {
        const bool dx_blocked = p.blk && gemm_blocked_supported(p.dtype, TB, p.in_dim[l]);   // reads W in place
        if ((l > 0 || p.V > 0) && !dx_blocked)
            LSTM_TRY(transpose_lp(p.dtype, par + p.off_W[l] * es, p.in_dim[l], wT + p.wT_off[l], p.G, p.G, p.in_dim[l], s));
        if (p.dtype == LSTM_DTYPE_FP32)   // the 16-bit path packs U^T per layer instead
            LSTM_TRY(transpose_lp(p.dtype, par + p.off_U[l] * es, p.H, wT + p.uT_off[l], p.G, p.G, p.H, s));
    }

    // head: dz = S * dloss/dz; gradients of the head and the seed for the top layer
    int cur = 0;
    char *dh_above = at(scratch, p.s_dh[cur]);
    const char *top = at(reserve, p.r_h[p.L - 1]) + (size_t)BH * es;
    if (p.head == LSTM_HEAD_FC_HINGE) {
        const char *act = at(reserve, p.r_fc);                 // relu(h W_fc^T + b_fc), [TB, F]
        char *dpre = at(scratch, p.s_fcd);                     // gradient before the ReLU, [TB, F]
        const char *Wfc = par + p.off_Wfc * es;
        LSTM_TRY(colsum(p.dtype, act, p.F, TB, p.F, dzu, loss_scale, colpart, grd + p.off_wh * es, s));
        LSTM_TRY(head_backward_dh(p.dtype, dzu, par + p.off_wh * es, loss_scale, act, dpre, TB, p.F, s));
        LSTM_TRY(colsum(p.dtype, dpre, p.F, TB, p.F, nullptr, nullptr, colpart, grd + p.off_bfc * es, s));
        // dW_fc = dpre^T h_top, contracted over all T*B rows
        GemmArgs w{};
        w.M = p.F; w.N = p.H; w.K = TB; w.ldc = p.H;
        w.C = grd + p.off_Wfc * es; w.out_lp = 1;
        w.splitk_ws = splitk; w.splits = p.split_fc; w.kclass = KC_GEMM_BATCHED;
        GemmArgs wt = w;
        wt.A = dpre; wt.lda = p.F; wt.B = top; wt.ldb = p.H;
        if (gemm_tn_supported(p.dtype, wt)) {
            LSTM_TRY(gemm_tn(p.dtype, wt, s));
        } else {
            char *dpreT = at(scratch, p.s_fcdT);
            char *topT = at(scratch, p.s_xT);
            LSTM_TRY(transpose_lp(p.dtype, dpre, p.F, dpreT, TB, TB, p.F, s));
            LSTM_TRY(transpose_lp(p.dtype, top, p.H, topT, TB, TB, p.H, s));
            w.A = dpreT; w.B = topT; w.lda = TB; w.ldb = TB;
            LSTM_TRY(gemm_nt(p.dtype, w, s));
        }
        // seed of the top LSTM layer: dh = dpre W_fc
        char *wfcT = at(scratch, p.s_fcwT);
        LSTM_TRY(transpose_lp(p.dtype, Wfc, p.H, wfcT, p.F, p.F, p.H, s));
        GemmArgs d{};
        d.A = dpre; d.B = wfcT; d.C = dh_above;
        d.M = TB; d.N = p.H; d.K = p.F;
        d.lda = p.F; d.ldb = p.F; d.ldc = p.H;
        d.out_lp = 1; d.kclass = KC_GEMM_BATCHED;
        LSTM_TRY(gemm_nt(p.dtype, d, s));
    } else if (p.head == LSTM_HEAD_LAST_BCE) {
        LSTM_TRY(fill_u32(dh_above, 0, (int64_t)(((size_t)TB * p.H * es + 3) / 4), s));
        const char *top_last = top + (size_t)(p.T - 1) * BH * es;
        LSTM_TRY(head_backward_dh(p.dtype, dzu, par + p.off_wh * es, loss_scale, nullptr, dh_above + (size_t)(p.T - 1) * BH * es, p.B, p.H, s));
        LSTM_TRY(colsum(p.dtype, top_last, p.H, p.Bw, p.H, dzu, loss_scale, colpart, grd + p.off_wh * es, s, p.W, p.Bw, p.P));
    } else {
        LSTM_TRY(head_backward_dh(p.dtype, dzu, par + p.off_wh * es, loss_scale, nullptr, dh_above, TB, p.H, s));
        LSTM_TRY(colsum(p.dtype, top, p.H, TB / p.W, p.H, dzu, loss_scale, colpart, grd + p.off_wh * es, s, p.W, p.Bw, p.P));
    }
    LSTM_TRY(head_backward_bias(p.dtype, dzu, loss_scale, p.head_rows / p.W, grd + p.off_bh * es, s, p.W, p.Bw, p.P));

    auto dA_rowmajor_needed = [&](int l) { return p.dA_rowmajor_needed(l); };
    if (p.wb) {
        // BPTT along anti-diagonals: cell (l, t) needs dA_{l,t+1} U_l (its own layer, one step later) and
        // dA_{l+1,t} W_{l+1} (the layer above, same step), both products of cells on the diagonal before.
        // Per diagonal: one launch with the gate arithmetic of all its cells, one with their products.
        const RecurrentDims rd = recurrent_dims(p.B, p.H);
        SetupBatch setup;
        for (int l = 0; l < p.L; ++l) {
            setup.pack_u_backward(par + p.off_U[l] * es, at(scratch, p.s_wb_utpk[l]));
            if (l > 0 && (!p.lag || p.lag_sdx)) setup.pack_u_backward(par + p.off_W[l] * es, at(scratch, p.s_wb_wtpk[l]));
            if (l > 0 && p.lag && !p.lag_sdx)      // the chunked dX GEMMs read W in 64x64 blocks
                LSTM_TRY(pack_blocked(p.dtype, par + p.off_W[l] * es, p.in_dim[l], p.G, p.in_dim[l], at(scratch, p.s_lag_wblk[l]), s));
            setup.zero(at(scratch, p.s_wb_dapk[l]), (int64_t)((rd.dapk_elems * es + 3) / 4));
            if (p.fb) setup.zero(at(scratch, p.s_wb_dapk1[l]), (int64_t)((rd.dapk_elems * es + 3) / 4));
            if (p.blk && !p.dA_packed_only(l)) setup.zero_pad(at(scratch, p.s_wb_dablk[l]), TB, p.G);
        }
        LSTM_TRY(setup.flush(p.dtype, p.B, p.H, s));
        if (p.fb) {
            // one launch per diagonal: every cell contracts over all 4H gate rows itself
            const int max_cells = fused_backward_max_cells();
            std::vector<FusedBackwardCell> fc;
            for (int d = 0; d < p.T + p.L - 1; ++d) {
                fc.clear();
                for (int l = p.L - 1; l >= 0; --l) {
                    const int t = p.T - 1 - (d - (p.L - 1 - l));
                    if (t < 0 || t >= p.T) continue;
                    auto dapk = [&](int layer, int step) { return at(scratch, (step & 1) ? p.s_wb_dapk1[layer] : p.s_wb_dapk[layer]); };
                    FusedBackwardCell c{};
                    const bool top_layer = l == p.L - 1, last = t == p.T - 1;
                    c.dApk_next = last ? nullptr : dapk(l, t + 1);
                    c.UTpk = last ? nullptr : at(scratch, p.s_wb_utpk[l]);
                    c.dApk_above = top_layer ? nullptr : dapk(l + 1, t);
                    c.WTpk = top_layer ? nullptr : at(scratch, p.s_wb_wtpk[l + 1]);
                    c.dh_above = top_layer ? dh_above + (size_t)t * BH * es : nullptr;
                    c.gates = at(reserve, p.r_gates[l]) + (size_t)t * p.B * p.G * es;
                    c.c_t = at(reserve, p.r_c[l]) + (size_t)(t + 1) * BH * es;
                    c.c_prev = at(reserve, p.r_c[l]) + (size_t)t * BH * es;
                    c.dc_state = (float *)at(scratch, p.s_wb_dc[l]);
                    c.dA = dA_rowmajor_needed(l) ? at(scratch, p.s_wb_dA[l]) + (size_t)t * p.B * p.G * es : nullptr;
                    c.dApk = dapk(l, t);
                    c.dAblk = p.blk ? at(scratch, p.s_wb_dablk[l]) + (size_t)t * (p.B / 64) * p.g_ncb * 4096 * es : nullptr;
                    c.first = last ? 1 : 0;
                    fc.push_back(c);
                }
                for (size_t i = 0; i < fc.size(); i += max_cells)
                    LSTM_TRY(backward_fused_wave(p.dtype, fc.data() + i, (int)std::min<size_t>(max_cells, fc.size() - i), p.g_ncb, p.B,
                                                 p.H, s));
            }
        }
        const int max_gates = wave_backward_max_gates(), max_gemms = p.lag ? tile_max_cells() : wave_backward_max_gemms();
        std::vector<WaveGates> gc;
        std::vector<WaveGemm> mm;
        // wide layers: layer l runs lag_c steps behind layer l + 1 and takes the gradient from above out of a
        // whole-sequence dX GEMM over the lag_c steps the layer above has just finished
        const int lag = p.lag ? p.lag_c : 1;
        const size_t slotg = p.blk ? (size_t)(p.B / 64) * p.g_ncb * 4096 * es : 0;   // bytes of one time slot of a blocked dA
        // first time step of the chunk that holds step t of a layer below the top (chunks count from the last step)
        auto chunk_lo = [&](int t) {
            const int k = p.T - 1 - t, t_hi = p.T - 1 - (k - k % lag);
            return t_hi - lag + 1 > 0 ? t_hi - lag + 1 : 0;
        };
        for (int d = 0; d < (p.fb ? 0 : p.T + (p.L - 1) * lag); ++d) {
            gc.clear(); mm.clear();
            for (int l = p.L - 2; p.lag && l >= 0; --l) {
                const int k = d - (p.L - 1 - l) * lag;
                if (k < 0 || k >= p.T || k % lag != 0) continue;
                const int t_hi = p.T - 1 - k, t_lo = chunk_lo(t_hi);
                if (p.lag_sdx) {
                    StreamGemmArgs g{};
                    g.A = at(scratch, p.s_lag_daseq[l + 1]) + (size_t)t_lo * rd.dapk_elems * es;
                    g.a_step_stride = (int64_t)rd.dapk_elems; g.rows_per_step = p.B;
                    g.B = at(scratch, p.s_wb_wtpk[l + 1]); g.gate_h = 0;
                    g.C = at(scratch, p.s_lag_dx[l]); g.ldc = p.H;
                    g.M = (t_hi - t_lo + 1) * p.B; g.N = p.H; g.K = p.G;
                    g.kclass = KC_GEMM_BATCHED;
                    LSTM_TRY(gemm_stream(p.dtype, g, s));
                    continue;
                }
                BlockedGemmArgs g{};
                g.A = BlockedOperand{at(scratch, p.s_wb_dablk[l + 1]) + (size_t)t_lo * slotg, p.g_ncb, 0};
                g.B = BlockedOperand{at(scratch, p.s_lag_wblk[l + 1]), (p.H + 63) / 64, 1};      // rows of W are the contraction index
                g.C = at(scratch, p.s_lag_dx[l]); g.ldc = p.H; g.out_lp = 1;
                g.M = (t_hi - t_lo + 1) * p.B; g.N = p.H; g.K = p.G;
                g.kclass = KC_GEMM_BATCHED;
                LSTM_TRY(gemm_blocked(p.dtype, g, s));
            }
            for (int l = p.L - 1; l >= 0; --l) {
                const int t = p.T - 1 - (d - (p.L - 1 - l) * lag);
                if (t < 0 || t >= p.T) continue;
                WaveGates c{};
                c.dh_above = l == p.L - 1 ? dh_above + (size_t)t * BH * es
                                          : (p.lag ? at(scratch, p.s_lag_dx[l]) + (size_t)(t - chunk_lo(t)) * BH * es : nullptr);
                c.above4 = (l < p.L - 1 && !p.lag) ? (const float *)at(scratch, p.s_wb_partW[l + 1]) : nullptr;
                c.partials = (const float *)at(scratch, p.s_wb_partU[l]);
                c.gates = at(reserve, p.r_gates[l]) + (size_t)t * p.B * p.G * es;
                c.c_t = at(reserve, p.r_c[l]) + (size_t)(t + 1) * BH * es;
                c.c_prev = at(reserve, p.r_c[l]) + (size_t)t * BH * es;
                c.dc_state = (float *)at(scratch, p.s_wb_dc[l]);
                c.dA = dA_rowmajor_needed(l) ? at(scratch, p.s_wb_dA[l]) + (size_t)t * p.B * p.G * es : nullptr;
                c.dApk = at(scratch, p.s_wb_dapk[l]);
                if (p.lag && p.lag_sdx && (l > 0 || p.lag_pk)) c.dApk = at(scratch, p.s_lag_daseq[l]) + (size_t)t * rd.dapk_elems * es;
                c.dAblk = (p.blk && !p.dA_packed_only(l)) ? at(scratch, p.s_wb_dablk[l]) + (size_t)t * slotg : nullptr;
                c.first = t == p.T - 1 ? 1 : 0;
                gc.push_back(c);
                if (t > 0) mm.push_back(WaveGemm{c.dApk, at(scratch, p.s_wb_utpk[l]), (float *)at(scratch, p.s_wb_partU[l])});
                if (l > 0 && !p.lag) mm.push_back(WaveGemm{c.dApk, at(scratch, p.s_wb_wtpk[l]), (float *)at(scratch, p.s_wb_partW[l])});
            }
            for (size_t i = 0; i < gc.size(); i += max_gates)
                LSTM_TRY(gates_backward_wave(p.dtype, gc.data() + i, (int)std::min<size_t>(max_gates, gc.size() - i), p.g_ncb, p.B,
                                             p.H, s, p.lag ? tile_backward_slices() : 4));
            for (size_t i = 0; i < mm.size(); i += max_gemms)
                LSTM_TRY((p.lag ? step_backward_gemm_tile : step_backward_gemm_wave)(p.dtype, mm.data() + i,
                                                                                     (int)std::min<size_t>(max_gemms, mm.size() - i), p.B, p.H, s));
        }
    }
    char *dAT = at(scratch, p.s_dAT);
    char *xT = at(scratch, p.s_xT);
    float *dh_rec = (float *)at(scratch, p.s_dhrec);
    float *dc_state = (float *)at(scratch, p.s_dcstate);
    for (int l = p.L - 1; l >= 0; --l) {
        const bool dA_rm = dA_rowmajor_needed(l);
        char *dA = at(scratch, p.wb ? p.s_wb_dA[l] : p.s_dA);
        const char *gates = at(reserve, p.r_gates[l]);
        const char *cs = at(reserve, p.r_c[l]);
        const char *hs = at(reserve, p.r_h[l]);
        const void *layer_in = l > 0 ? (const void *)(at(reserve, p.r_h[l - 1]) + (size_t)BH * es)
                                     : (p.V > 0 ? (const void *)at(reserve, p.r_xemb) : x);
        const int I = p.in_dim[l];
        const bool fused = p.dtype != LSTM_DTYPE_FP32;
        char *utpk = at(scratch, p.s_upk);
        char *dapk[2] = {at(scratch, p.s_apk[0]), at(scratch, p.s_apk[1])};
        if (fused && !p.wb) {
            const RecurrentDims rd = recurrent_dims(p.B, p.H);
            SetupBatch setup;
            setup.pack_u_backward(par + p.off_U[l] * es, utpk);
            for (int k = 0; k < 2; ++k) setup.zero(dapk[k], (int64_t)((rd.dapk_elems * es + 3) / 4));
            if (p.blk) setup.zero_pad(at(scratch, p.s_dablk), TB, p.G);
            LSTM_TRY(setup.flush(p.dtype, p.B, p.H, s));
        }
        const bool pk_only = p.dA_packed_only(l);
        char *dablk = (p.blk && !pk_only) ? at(scratch, p.wb ? p.s_wb_dablk[l] : p.s_dablk) : nullptr;
        const bool fused_step = fused && !p.wb && step_backward_fused_supported(p.dtype, p.B, p.H) && (dA_rm || dablk);
        const bool rows_bwd = fused && !p.wb && rows_backward_supported(p.dtype, p.B, p.H) && (dA_rm || dablk);
        // ... and adds up the bias gradient's parts on the way (each worker's rows are whole groups of 32)
        const bool rows_bias = rows_bwd && !dA_rm && (p.W == 1 || p.Bw % 32 == 0);
        if (rows_bwd) {
            // every workgroup walks its 32 rows back through all T steps: one launch for the layer
            RowsBackward r{};
            r.UTpk = utpk; r.dh_above = dh_above; r.gates = gates; r.cs = cs;
            r.dA = dA_rm ? dA : nullptr; r.dAblk = dablk;
            r.bias_partial = rows_bias ? colpart : nullptr;
            r.slot_blk = (int64_t)(p.B / 64) * p.g_ncb * 4096; r.blk_ncb = p.g_ncb;
            LSTM_TRY(rows_backward(p.dtype, r, p.T, p.B, p.H, s));
        }
        for (int t = (p.wb || rows_bwd) ? -1 : p.T - 1; t >= 0; --t) {      // along the diagonals the steps are already done
            const bool last = t == p.T - 1;
            if (fused && fused_step) {
                // thousands of rows per step: product and gate arithmetic in one launch, no partial sums in memory
                FusedBackwardCell c{};
                c.dApk_next = last ? nullptr : dapk[(t + 1) & 1];
                c.UTpk = last ? nullptr : utpk;
                c.dh_above = dh_above + (size_t)t * BH * es;
                c.gates = gates + (size_t)t * p.B * p.G * es;
                c.c_t = cs + (size_t)(t + 1) * BH * es;
                c.c_prev = cs + (size_t)t * BH * es;
                c.dc_state = dc_state;
                c.dA = dA_rm ? dA + (size_t)t * p.B * p.G * es : nullptr;
                c.dApk = dapk[t & 1];
                c.dAblk = dablk ? dablk + (size_t)t * (p.B / 64) * p.g_ncb * 4096 * es : nullptr;
                c.first = last ? 1 : 0;
                LSTM_TRY(step_backward_fused(p.dtype, c, p.g_ncb, p.B, p.H, s));
                continue;
            }
            if (fused) {
                // dA_{t+1} U as four per-gate K-slices, summed by the gate kernel
                float *part = (float *)at(scratch, p.s_part);
                if (!last) LSTM_TRY(step_backward_gemm(p.dtype, dapk[(t + 1) & 1], utpk, part, p.B, p.H, s));
                LSTM_TRY(gates_backward_packed(p.dtype, dh_above + (size_t)t * BH * es, part, gates + (size_t)t * p.B * p.G * es,
                                               cs + (size_t)(t + 1) * BH * es, cs + (size_t)t * BH * es, dc_state,
                                               dA_rm ? dA + (size_t)t * p.B * p.G * es : nullptr, dapk[t & 1],
                                               dablk ? dablk + (size_t)t * (p.B / 64) * p.g_ncb * 4096 * es : nullptr, p.g_ncb,
                                               p.B, p.H, last ? 1 : 0, s));
                continue;
            }
            if (!last) {
                // dh_rec = dA_{t+1} U   (contract over the 4H gate rows)
                GemmArgs r{};
                r.A = dA + (size_t)(t + 1) * p.B * p.G * es; r.B = wT + p.uT_off[l]; r.C = dh_rec;
                r.M = p.B; r.N = p.H; r.K = p.G;
                r.lda = p.G; r.ldb = p.G; r.ldc = p.H;
                r.kclass = KC_GEMM_STEP;
                LSTM_TRY(gemm_nt(p.dtype, r, s));
            }
            LSTM_TRY(gates_backward(p.dtype, dh_above + (size_t)t * BH * es, last ? nullptr : dh_rec,
                                    gates + (size_t)t * p.B * p.G * es, cs + (size_t)(t + 1) * BH * es,
                                    cs + (size_t)t * BH * es, dc_state, dA + (size_t)t * p.B * p.G * es, p.B, p.H,
                                    last ? 1 : 0, 1, s));
        }
        char *d_below = at(scratch, p.s_dh[cur ^ 1]);
        // blocked operands of this layer: dA (written by the gate kernel), its input sequence and W
        BlockedOperand in_blk{nullptr, 0, 0};
        char *wblk = p.blk ? at(scratch, p.s_wblk) : nullptr;
        if (p.blk) {
            if (l == 0) in_blk = BlockedOperand{at(reserve, p.r_xblk), (p.in_dim[0] + 63) / 64, 0, p.lag_x0 ? 1 : 0};
            else in_blk = BlockedOperand{at(reserve, p.r_hblk[l - 1]) + (size_t)(p.B / 64) * p.h_ncb * 4096 * es, p.h_ncb, 0, p.lag_pk ? 1 : 0};
        }
        if ((l > 0 && !p.wb) || (l == 0 && p.V > 0)) {
            // dX = dA W  for the layer below (or the embedding rows); along the diagonals the layers
            // above the first got theirs step by step
            if (p.blk && gemm_blocked_supported(p.dtype, TB, I)) {
                LSTM_TRY(pack_blocked(p.dtype, par + p.off_W[l] * es, I, p.G, I, wblk, s));
                BlockedGemmArgs d{};
                d.A = BlockedOperand{dablk, p.g_ncb, 0};
                d.B = BlockedOperand{wblk, (I + 63) / 64, 1};        // rows of W are the contraction index
                d.C = d_below; d.ldc = I; d.out_lp = 1;
                d.M = TB; d.N = I; d.K = p.G;
                d.kclass = KC_GEMM_BATCHED;
                LSTM_TRY(gemm_blocked(p.dtype, d, s));
            } else {
                GemmArgs d{};
                d.A = dA; d.B = wT + p.wT_off[l]; d.C = d_below;
                d.M = TB; d.N = I; d.K = p.G;
                d.lda = p.G; d.ldb = p.G; d.ldc = I;
                d.out_lp = 1; d.kclass = KC_GEMM_BATCHED;
                LSTM_TRY(gemm_nt(p.dtype, d, s));
            }
        }
        // weight gradients dW = dA^T X and dU = dA^T H_prev, contracted over all T*B rows with
        // fp32 accumulation.  Preferred: blocked operands read as they lie in memory (rows are
        // the contraction index); then the row-major form of the same kernel; otherwise explicit
        // transposes feed the K-contiguous kernel.
        GemmArgs w{};
        w.M = p.G; w.N = I; w.K = TB; w.ldc = I;
        w.C = grd + p.off_W[l] * es;
        w.kclass = KC_GEMM_BATCHED;
        w.out_lp = 1; w.splitk_ws = splitk; w.splits = p.split_w[l];
        GemmArgs u = w;
        u.N = p.H; u.ldc = p.H;
        u.C = grd + p.off_U[l] * es;
        u.splits = p.split_u[l];
        GemmArgs wt = w, ut = u;
        wt.A = dA; wt.lda = p.G; wt.B = layer_in; wt.ldb = I;
        ut.A = dA; ut.lda = p.G; ut.B = hs; ut.ldb = p.H;                 // h_0..h_{T-1}
        // dW: always the blocked kernel when the blocked copies exist, whatever the input width (a narrow
        // input wastes part of a tile, the alternative is two transposes); several workers need it anyway
        // (its per-worker K mapping)
        const bool w_blk = p.blk;
        const bool u_blk = p.blk && (p.W > 1 || gemm_blocked_supported(p.dtype, p.G, p.H));
        const bool w_tn = !w_blk && gemm_tn_supported(p.dtype, wt), u_tn = !u_blk && gemm_tn_supported(p.dtype, ut);
        if ((!w_blk && !w_tn) || (!u_blk && !u_tn)) LSTM_TRY(transpose_lp(p.dtype, dA, p.G, dAT, TB, TB, p.G, s));
        auto blocked_wgrad = [&](const GemmArgs &r, const BlockedOperand &bop) {
            BlockedGemmArgs g{};
            // both operands blocked, or both the packed per-step copies
            g.A = bop.packed ? BlockedOperand{at(scratch, p.s_lag_daseq[l]), p.g_ncb, 1, 1} : BlockedOperand{dablk, p.g_ncb, 1, 0};
            g.B = BlockedOperand{bop.ptr, bop.ncb, 1, bop.packed};
            g.C = r.C; g.ldc = r.ldc; g.out_lp = 1;
            g.M = r.M; g.N = r.N; g.K = r.K;
            g.splitk_ws = r.splitk_ws; g.splits = r.splits; g.kclass = r.kclass;
            if (p.W > 1) {
                // one product per worker over that worker's rows of every time step
                g.K = r.K / p.W;
                g.batch = p.W; g.seg_len = p.Bw / 64; g.seg_stride = p.B / 64; g.batch_c = p.P;
                g.splitk_ws = nullptr; g.splits = 1;
            }
            // large single products: the hand-scheduled kernel
            if (p.W == 1 && gemm_stream_tn_supported(p.dtype, g)) return gemm_stream_tn(p.dtype, g, s);
            return gemm_blocked(p.dtype, g, s);
        };
        // several workers: dW and dU of a layer in one launch (they share dA, which then comes from memory once)
        const bool wu_together = p.W > 1 && w_blk && u_blk && (p.G + 255) / 256 <= 8;
        if (wu_together) {
            BlockedGemmArgs g{};
            g.A = BlockedOperand{dablk, p.g_ncb, 1, 0};
            g.B = BlockedOperand{in_blk.ptr, in_blk.ncb, 1, 0};
            g.C = w.C; g.ldc = w.ldc; g.out_lp = 1;
            g.M = w.M; g.N = w.N; g.K = w.K / p.W;
            g.B2 = BlockedOperand{at(reserve, p.r_hblk[l]), p.h_ncb, 1, 0};
            g.C2 = u.C; g.ldc2 = u.ldc; g.N2 = u.N;
            g.batch = p.W; g.seg_len = p.Bw / 64; g.seg_stride = p.B / 64; g.batch_c = p.P;
            g.kclass = w.kclass;
            LSTM_TRY(gemm_blocked(p.dtype, g, s));
        } else if (w_blk) {
            LSTM_TRY(blocked_wgrad(w, in_blk));
        } else if (w_tn) {
            LSTM_TRY(gemm_tn(p.dtype, wt, s));
        } else {
            LSTM_TRY(transpose_lp(p.dtype, layer_in, I, xT, TB, TB, I, s));
            w.A = dAT; w.B = xT; w.lda = TB; w.ldb = TB;
            LSTM_TRY(gemm_nt(p.dtype, w, s));
        }
        if (wu_together) {
            // (done above)
        } else if (u_blk) {
            LSTM_TRY(blocked_wgrad(u, BlockedOperand{at(reserve, p.r_hblk[l]), p.h_ncb, 1, p.lag_pk ? 1 : 0}));
        } else if (u_tn) {
            LSTM_TRY(gemm_tn(p.dtype, ut, s));
        } else {
            LSTM_TRY(transpose_lp(p.dtype, hs, p.H, xT, TB, TB, p.H, s));
            u.A = dAT; u.B = xT; u.lda = TB; u.ldb = TB;
            LSTM_TRY(gemm_nt(p.dtype, u, s));
        }
        if (dA_rm) LSTM_TRY(colsum(p.dtype, dA, p.G, TB / p.W, p.G, nullptr, nullptr, colpart, grd + p.off_b[l] * es, s, p.W, p.Bw, p.P));
        else if (rows_bias) LSTM_TRY(colsum_finish(p.dtype, colpart, p.W == 1 ? rows_backward_groups(p.B) : p.Bw / 32, p.G, grd + p.off_b[l] * es, s, p.W, p.P));
        else if (pk_only) LSTM_TRY(colsum_blocked(p.dtype, at(scratch, p.s_lag_daseq[l]), p.g_ncb, TB, p.G, colpart, grd + p.off_b[l] * es, s, 1, 0, 0, 1));
        else LSTM_TRY(colsum_blocked(p.dtype, dablk, p.g_ncb, TB / p.W, p.G, colpart, grd + p.off_b[l] * es, s, p.W, p.Bw, p.P));
        cur ^= 1;
        dh_above = d_below;
    }
    if (p.V > 0) {
        float *dE32 = (float *)at(scratch, p.s_dE32);
        LSTM_TRY(fill_u32(dE32, 0, (int64_t)p.V * p.D, s));
        LSTM_TRY(embed_scatter_add(p.dtype, (const int32_t *)x, dh_above, dE32, TB, p.V, p.D, s));
        LSTM_TRY(cast_f32_to_lp(p.dtype, dE32, grd + p.off_E * es, (int64_t)p.V * p.D, s));
    }
    return LSTM_OK;
}

// ---- lstm_forward for callers that cannot allocate: the scratch workspace lives in the library's own
// device image.  Every GPU the library runs on holds its own copy of the array at its own address;
// the address is looked up once per device and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char static_scratch[LSTM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kMaxDevices] = {};

int static_scratch_address(void **out) {
    int dev = -1;
    LSTM_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device index %d outside the range this build keeps static scratch addresses for", dev);
        return LSTM_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        LSTM_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)));
        if (!ptr) {
            set_error("hipGetSymbolAddress returned a null address for the static scratch array");
            return LSTM_ERR_HIP;
        }
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return LSTM_OK;
}
}  // namespace

extern "C" int lstm_forward_static_scratch(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                                           const void *h0, const float *c0, void *reserve, size_t reserve_bytes, float *loss,
                                           void *hT, float *cT, void *stream) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    if (p.scratch_bytes > (size_t)LSTM_STATIC_SCRATCH_BYTES) {
        set_error("lstm_forward_static_scratch: this config needs %zu bytes of scratch, the built-in buffer holds %zu; "
                  "use lstm_forward with a caller-provided scratch buffer",
                  p.scratch_bytes, (size_t)LSTM_STATIC_SCRATCH_BYTES);
        return LSTM_ERR_WORKSPACE;
    }
    void *scratch_ptr = nullptr;
    LSTM_TRY(static_scratch_address(&scratch_ptr));
    // same kernels, same order as lstm_forward; every scratch element a kernel reads is written by the
    // library first, so what an earlier call left behind in the array never enters a result
    return lstm_forward(cfg, params_lp, x, targets, h0, c0, reserve, reserve_bytes, scratch_ptr, (size_t)LSTM_STATIC_SCRATCH_BYTES,
                        loss, hT, cT, stream);
}

// Step 11 of the iteration taken on its own: the working copy as the round-to-nearest-even cast of the
// fp32 master weights (what master_update leaves behind after every step), for the first step.
extern "C" int lstm_cast_params(int64_t n_params, const float *master, void *params_lp_out, int32_t dtype, void *stream) {
    if (n_params < 1 || dtype < LSTM_DTYPE_FP32 || dtype > LSTM_DTYPE_BF16) {
        set_error("lstm_cast_params: bad n_params %lld or dtype %d", (long long)n_params, dtype);
        return LSTM_ERR_INVALID;
    }
    LSTM_TRY(check_ptr(master, "master"));
    LSTM_TRY(check_ptr(params_lp_out, "params_lp_out"));
    return cast_f32_to_lp(dtype, master, params_lp_out, n_params, (hipStream_t)stream);
}

// Diagnostic: the regions of the workspace plan, for overlap checks on the host.
extern "C" int lstm_debug_plan_regions(const lstm_config *cfg, int32_t max_regions, int32_t *which, size_t *offsets,
                                       size_t *bytes, int32_t *count) {
    Plan p;
    LSTM_TRY(make_plan(cfg, p));
    if (!count || (max_regions > 0 && (!which || !offsets || !bytes))) {
        set_error("lstm_debug_plan_regions: null output");
        return LSTM_ERR_INVALID;
    }
    *count = (int32_t)p.regions.size();
    for (int i = 0; i < (int)p.regions.size() && i < max_regions; ++i) {
        which[i] = p.regions[i].which; offsets[i] = p.regions[i].offset; bytes[i] = p.regions[i].bytes;
    }
    return LSTM_OK;
}

// Diagnostic: one whole-sequence GEMM through the same dispatch the training step uses.
// layout 0: C = A B^T, row-major A[M,K], B[N,K];  1: C = A^T B, row-major A[K,M], B[K,N];
// 2/3/4: operands in 64x64 blocks (see pack_blocked), roles (A,B) = (rows M, rows N) /
// (rows M, rows K) / (rows K, rows K); 5: as 4 on the kernel of gemm_stream.hip; 6: as 5 with every block in fragment order.  C is row-major lp [M,N].
extern "C" int lstm_debug_gemm(int32_t dtype, int32_t layout, int32_t M, int32_t N, int32_t K, const void *A, const void *B,
                               void *C, float *splitk_ws, int32_t splits, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    if (layout <= 1) {
        GemmArgs g{};
        g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K;
        g.lda = layout == 0 ? K : M; g.ldb = layout == 0 ? K : N; g.ldc = N;
        g.out_lp = 1; g.splitk_ws = splitk_ws; g.splits = splits; g.kclass = KC_GEMM_BATCHED;
        return layout == 0 ? gemm_nt(dtype, g, s) : gemm_tn(dtype, g, s);
    }
    BlockedGemmArgs g{};
    const int ta = layout >= 4, tb = layout >= 3;
    g.A = BlockedOperand{A, ((ta ? M : K) + 63) / 64, ta};
    g.B = BlockedOperand{B, ((tb ? N : K) + 63) / 64, tb};
    g.C = C; g.ldc = N; g.out_lp = 1; g.M = M; g.N = N; g.K = K;
    g.splitk_ws = splitk_ws; g.splits = splits; g.kclass = KC_GEMM_BATCHED;
    if (layout == 6) g.A.packed = g.B.packed = 1;
    return layout >= 5 ? gemm_stream_tn(dtype, g, s) : gemm_blocked(dtype, g, s);
}

// Diagnostic: the whole-sequence GEMM on operands in packed (MFMA-fragment) order.
extern "C" int lstm_debug_gemm_stream(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t rows_per_step, int64_t a_step_stride,
                                      int32_t gate_h, const void *A, const void *B, const void *bias, void *C, void *stream) {
    StreamGemmArgs g{};
    g.A = A; g.a_step_stride = a_step_stride; g.rows_per_step = rows_per_step; g.B = B; g.C = C; g.ldc = N; g.bias = bias;
    g.M = M; g.N = N; g.K = K; g.gate_h = gate_h; g.kclass = KC_GEMM_BATCHED;
    return gemm_stream(dtype, g, (hipStream_t)stream);
}

// Diagnostic: register-resident MFMA loop on caller-provided operand values.
extern "C" int lstm_debug_mfma_rate(int32_t dtype, const void *operands, int32_t iters, float *sink, double *flops,
                                    void *stream) {
    return mfma_rate(dtype, operands, iters, sink, flops, (hipStream_t)stream);
}

// Diagnostic: row-major [rows, cols] -> 64x64 blocks.
extern "C" int lstm_debug_pack_blocked(int32_t dtype, const void *src, int32_t rows, int32_t cols, void *dst, void *stream) {
    return pack_blocked(dtype, src, cols, rows, cols, dst, (hipStream_t)stream);
}

