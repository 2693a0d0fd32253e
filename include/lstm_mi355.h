/*
 * lstm_mi355.h — C ABI of the MI355X (gfx950) mixed-precision stacked-LSTM
 * training step.
 *
 * One data-parallel worker's iteration as the paper states it (Section
 * "Neural Network architecture": fprop, loss, bprop by BPTT, weight update;
 * Section "Distributed computing framework", steps 3-5): forward through
 * time, loss, backward through time on the loss multiplied by a scale
 * (Section "Performance evaluation", Eq. 6), averaging of the workers' raw
 * gradients, the worker-count learning-rate schedule (Section "Learning rate
 * schedule", Eq. 3-4) and the momentum update of Eq. 1-2 on fp32 master
 * weights with a re-cast to the low-precision working copy.
 *
 * Conventions (all entry points)
 *   - every pointer named below as "device" is a GPU global-memory address on
 *     the current HIP device; "host" pointers are ordinary CPU memory.
 *   - the caller owns every buffer; the library only borrows pointers for the
 *     duration of the work it enqueues.  Nothing is allocated or freed on the
 *     device and no call synchronises with the host: all kernels are enqueued
 *     on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - return value: LSTM_OK or a negative status; the text of the last error
 *     on the calling thread is available from lstm_last_error().
 *   - "lp" is the storage type selected by lstm_config.dtype (fp32, IEEE
 *     half, or bfloat16); accumulation is always fp32.
 *   - device buffers must be 16-byte aligned (grads_lp of lstm_backward, which
 *     may be one row of a worker-major [N,P] matrix, only to its element size).
 *   - sequences are time-major: x is [T,B,I], row (t*B + b).
 *   - calls that share a reserve/scratch buffer must be ordered on one
 *     stream; distinct buffers on distinct streams may overlap.
 */
#ifndef LSTM_MI355_H
#define LSTM_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LSTM_ABI_VERSION 4

enum {
    LSTM_OK = 0,
    LSTM_ERR_INVALID = -1,      /* null pointer, misaligned buffer, bad enum or size */
    LSTM_ERR_UNSUPPORTED = -2,  /* shape or dtype this build has no kernel for */
    LSTM_ERR_WORKSPACE = -3,    /* reserve_bytes / scratch_bytes below what lstm_workspace_bytes reports for the config */
    LSTM_ERR_HIP = -4           /* a HIP runtime call failed */
};

enum { LSTM_DTYPE_FP32 = 0, LSTM_DTYPE_FP16 = 1, LSTM_DTYPE_BF16 = 2 };

enum {
    LSTM_HEAD_STEP_BCE = 1,  /* z[t,b] = w.h_top[t,b] + b0, sigmoid + binary cross-entropy, every step */
    LSTM_HEAD_LAST_BCE = 2,  /* same, last time step only (targets [B,1])                            */
    LSTM_HEAD_STEP_MSE = 3,  /* z[t,b] linear, squared error, every step                             */
    LSTM_HEAD_FC_HINGE = 4   /* the head of Fig. 2: a[t,b] = relu(W_fc h_top[t,b] + b_fc) (head_hidden units),
                                z[t,b] = w.a[t,b] + b0, hinge loss max(0, 1 - y z) with targets y = +-1 (Eq. 6
                                without its multiplier, which is lstm_backward's loss scale), every step;
                                derivative 0 at the kink */
};

enum { LSTM_OPT_SGD_MOMENTUM = 0, LSTM_OPT_ADAM = 1 };

/* tensor kinds for lstm_param_offset */
enum { LSTM_P_EMBED = 0, LSTM_P_W = 1, LSTM_P_U = 2, LSTM_P_B = 3, LSTM_P_HEAD_W = 4, LSTM_P_HEAD_B = 5,
       LSTM_P_FC_W = 6, LSTM_P_FC_B = 7 };

/* Model shape.  Fig. 2 of the paper: stacked LSTM layers of `hidden` units over
 * (batch, sequence length, feature) inputs with one output per time slice. */
typedef struct {
    int32_t num_layers;  /* L >= 1                                              */
    int32_t input_dim;   /* I, feature dimension of x (ignored when vocab > 0)  */
    int32_t hidden;      /* H                                                   */
    int32_t seq_len;     /* T                                                   */
    int32_t batch;       /* B                                                   */
    int32_t dtype;       /* LSTM_DTYPE_*: storage of weights/activations/grads  */
    int32_t head;        /* LSTM_HEAD_*                                         */
    int32_t out_dim;     /* must be 1                                           */
    int32_t vocab;       /* > 0: x holds int32 token ids, looked up in E[V,D]   */
    int32_t embed_dim;   /* D (input dim of layer 0 when vocab > 0)             */
    int32_t head_hidden; /* F >= 1 with LSTM_HEAD_FC_HINGE, ignored otherwise   */
    int32_t workers;     /* W: simulated workers processed together, each with
                            its own micro-batch of `batch` samples (0 reads as
                            1).  With W > 1: x is [T, W, B, I], targets
                            [T, W, B, 1] (last-step head: [W, B, 1]), h0/c0/
                            hT/cT [L, W*B, H], loss fp32[W] (one mean per
                            worker), grads_lp lp[W, n_params] (one raw
                            gradient per worker, as if each had run alone).
                            All workers share params_lp.  Supported for the
                            16-bit types, batch a multiple of 64, no
                            embedding, the three single-layer heads;
                            otherwise LSTM_ERR_UNSUPPORTED (call once per
                            worker instead).                                   */
} lstm_config;

/* Optimiser and loss-scale policy for master_update. */
typedef struct {
    int32_t kind;            /* LSTM_OPT_*                                           */
    float momentum;          /* m of Eq. 1 (SGD)                                     */
    float beta1, beta2, eps; /* Adam                                                 */
    float weight_decay;      /* g <- g + wd * W before the update                    */
    int32_t dynamic_scale;   /* 0: loss scale never changes; 1: halve/grow policy    */
    float scale_backoff;     /* factor applied after an overflowed step (0.5)        */
    float scale_growth;      /* factor applied after growth_interval clean steps (2) */
    int32_t growth_interval; /* clean steps in a row before the scale grows          */
} optimizer_config;

int lstm_abi_version(void);

/* Text of the most recent error on this thread ("" if none).  Host memory owned
 * by the library, valid until the next failing call on the same thread. */
const char *lstm_last_error(void);

/* Number of elements of the flat parameter vector.  Layout (all row-major):
 *   [E[V,D]]  then for l = 0..L-1: W_l[4H,I_l], U_l[4H,H], b_l[4H]  then
 *   w_head[H], b_head[1];  I_0 = input_dim (or D), I_l = H above.
 *   With LSTM_HEAD_FC_HINGE the tail is W_fc[F,H], b_fc[F], w_head[F], b_head[1].
 * The 4H rows are grouped by gate in the order input, forget, cell candidate,
 * output.  Gradient buffers use the same layout.  n_params: host, out. */
int lstm_param_count(const lstm_config *cfg, int64_t *n_params);

/* Element offset and element count of one tensor inside the flat vector.
 * kind = LSTM_P_*; layer is ignored for the embedding and head tensors.
 * offset, count: host, out. */
int lstm_param_offset(const lstm_config *cfg, int32_t kind, int32_t layer, int64_t *offset, int64_t *count);

/* Bytes the caller must provide for `reserve` (activations saved by
 * lstm_forward for lstm_backward) and `scratch` (temporaries of either call).
 * Both host, out. */
int lstm_workspace_bytes(const lstm_config *cfg, size_t *reserve_bytes, size_t *scratch_bytes);

/* fprop + loss (Section "Neural Network architecture").
 *   params_lp : device, lp[n_params], the working copy of the weights.
 *   x         : device, lp[T,B,I], or int32[T,B] token ids when vocab > 0
 *               (ids must lie in [0,vocab); out-of-range ids are clamped).
 *   targets   : device, fp32 [T,B,1] (per-step heads) or [B,1] (last-step).
 *   h0, c0    : device or NULL (= zeros). h0: lp[L,B,H]; c0: fp32[L,B,H].
 *   reserve   : device, out; consumed by lstm_backward.
 *   scratch   : device, contents undefined afterwards.
 *   reserve_bytes, scratch_bytes : sizes of the two buffers as allocated by the caller; when either is
 *               below what lstm_workspace_bytes reports for cfg the call returns LSTM_ERR_WORKSPACE and
 *               enqueues nothing (a config edited after sizing the buffers selects other kernels and
 *               another layout).
 *   loss      : device, out, one fp32: mean of the per-output loss (unscaled).
 *   hT, cT    : device or NULL, out; final states, same shapes/types as h0, c0.
 * Per layer and step: a = W x_t + U h_{t-1} + b; i,f,o = logistic, g = tanh;
 * c_t = f c_{t-1} + i g; h_t = o tanh(c_t). */
int lstm_forward(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                 const void *h0, const float *c0, void *reserve, size_t reserve_bytes, void *scratch,
                 size_t scratch_bytes, float *loss, void *hT, float *cT, void *stream);

/* lstm_forward for callers that cannot allocate device memory or pass a workspace along: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as lstm_forward, except that the scratch workspace is a buffer of
 * LSTM_STATIC_SCRATCH_BYTES built into the library's device image (one copy per GPU, held until the
 * process ends); the call allocates and frees nothing.  A config whose scratch requirement
 * (lstm_workspace_bytes) exceeds that size is refused with LSTM_ERR_WORKSPACE.  All calls on one GPU
 * share the buffer: calls that overlap in time on the same GPU (different streams or threads) race;
 * order them on one stream.  The buffer keeps the last call's contents, which never enter a result
 * (every element a kernel reads was written by the same call first). */
#define LSTM_STATIC_SCRATCH_BYTES (32u << 20)
int lstm_forward_static_scratch(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                                const void *h0, const float *c0, void *reserve, size_t reserve_bytes, float *loss,
                                void *hT, float *cT, void *stream);

/* bprop by BPTT of (loss_scale * loss) (Section "Performance evaluation",
 * Eq. 6: the scalar multiplies the loss before the partial derivatives).
 *   params_lp, x, targets, reserve : as given to / produced by lstm_forward.
 *   reserve_bytes, scratch_bytes   : as for lstm_forward (LSTM_ERR_WORKSPACE when too small).
 *   loss_scale : device, one fp32 (read on the device, no host sync).
 *   grads_lp   : device, out, lp[n_params] = loss_scale * dloss/dtheta in the
 *                parameter layout; half-precision overflow shows up as Inf.
 * Weight gradients are accumulated over all time steps in fp32 and rounded to
 * lp once. */
int lstm_backward(const lstm_config *cfg, const void *params_lp, const void *x, const float *targets,
                  const void *reserve, size_t reserve_bytes, void *scratch, size_t scratch_bytes,
                  const float *loss_scale, void *grads_lp, void *stream);

/* Step 4 of the framework list: sum the workers' raw gradients, divide by the
 * number of workers, and undo the loss scale; also report Inf/NaN.
 *   grads_lp   : device, lp[n_workers, n_params] contiguous (dtype = LSTM_DTYPE_*).
 *   loss_scale : device, one fp32.
 *   avg_grad   : device, out, fp32[n_params] = sum_w g_w / (n_workers * scale).
 *   found_inf  : device, out, one int32: 1 if any input element is Inf/NaN else 0.
 * Reads low precision, accumulates in fp32. */
int grad_average(int64_t n_params, int32_t n_workers, const void *grads_lp, int32_t dtype,
                 const float *loss_scale, float *avg_grad, int32_t *found_inf, void *stream);

/* Fault-tolerant form of step 4 (Section "Distributed computing framework", last paragraph:
 * the master proceeds once a fraction of the workers, normally 90-95 %, has delivered).
 * Only the gradients of the workers that reported enter the average and the Inf/NaN test;
 * the rows of the others are never read.  Whether enough workers have reported is the
 * caller's decision, taken before the call.
 *   participating   : device, int32[n_workers], non-zero = this worker's gradient is present.
 *   avg_grad        : device, out, fp32[n_params] = sum over present w of g_w / (n_present * scale);
 *                     all zero when nobody is present.
 *   n_participating : device, out, one int32 = n_present (may be NULL).
 * Everything else as grad_average. */
int grad_average_masked(int64_t n_params, int32_t n_workers, const void *grads_lp, int32_t dtype,
                        const float *loss_scale, const int32_t *participating, float *avg_grad,
                        int32_t *found_inf, int32_t *n_participating, void *stream);

/* Step 5: optimiser state and global weights (Eq. 1-2:  H <- m H - lr g,
 * W <- W + H) on fp32 master weights, then round to the lp working copy.
 *   lr         : learning rate for this iteration (see lr_schedule).
 *   step       : 1-based iteration count (Adam bias correction only).
 *   master     : device, in/out, fp32[n_params].
 *   state1     : device, in/out, fp32[n_params]: H (SGD) or first moment (Adam).
 *   state2     : device, in/out, fp32[n_params]: second moment (Adam); NULL for SGD.
 *   avg_grad   : device, fp32[n_params], unscaled averaged gradient.
 *   found_inf  : device, one int32 from grad_average.  When it is 1 the step is
 *                skipped: master, state and params_lp_out keep their bits.
 *   loss_scale, good_steps : device, in/out, one fp32 / one int32.  With
 *                dynamic_scale: overflow -> scale *= backoff, good_steps = 0;
 *                else good_steps += 1 and after growth_interval clean steps
 *                scale *= growth.  Untouched when dynamic_scale = 0.
 *   params_lp_out : device, out, lp[n_params] (dtype) rounded to nearest even. */
int master_update(int64_t n_params, const optimizer_config *opt, float lr, int64_t step, float *master,
                  float *state1, float *state2, const float *avg_grad, const int32_t *found_inf,
                  float *loss_scale, int32_t *good_steps, void *params_lp_out, int32_t dtype, void *stream);

/* The last action of step 5 taken on its own: params_lp_out = round-to-nearest-even cast of the fp32
 * master weights to the working type, which is what master_update leaves behind after every
 * iteration.  For the first iteration, before any update has run.
 *   master        : device, fp32[n_params].
 *   params_lp_out : device, out, lp[n_params] (dtype = LSTM_DTYPE_*). */
int lstm_cast_params(int64_t n_params, const float *master, void *params_lp_out, int32_t dtype, void *stream);

/* Section "Learning rate schedule" (host, pure function).
 *   base = lr0 / (1 + n_workers / n_half)                      (Eq. 4)
 *   if base * n_workers > eff_lr_max: base = eff_lr_max / n_workers
 *   index < warmup_steps : base * (index + 1) / warmup_steps
 *   otherwise            : base * gamma^(index - warmup_steps + 1), or
 *                          base * gamma^index when warmup_steps = 0   (Eq. 3)
 * Returns 0 for invalid arguments (n_workers < 1, n_half <= 0). */
float lr_schedule(float lr0, int32_t n_workers, float n_half, float eff_lr_max, int32_t warmup_steps,
                  float gamma, int64_t index);

#ifdef __cplusplus
}
#endif
#endif /* LSTM_MI355_H */
