// HBM-bound kernels of the exchange/update half of the step:
//   grad_average  - sum N workers' low-precision gradients in fp32, divide by
//                   N and by the loss scale, flag Inf/NaN (wavefront vote, one
//                   atomic per wavefront that saw one).
//   master_update - momentum SGD of Eq. 1-2 (or Adam) on fp32 master weights,
//                   skipped on overflow, fused with the cast to the working copy.
#include "kernels.h"

#include <math.h>

namespace lstm {
namespace {

template <typename T> struct Bits;
template <> struct Bits<_Float16> {
    __device__ static inline bool nonfinite(uint16_t b) { return (b & 0x7c00u) == 0x7c00u; }
    __device__ static inline float to_f(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
};
template <> struct Bits<bf16_t> {
    __device__ static inline bool nonfinite(uint16_t b) { return (b & 0x7f80u) == 0x7f80u; }
    __device__ static inline float to_f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
};

struct __attribute__((packed, aligned(2))) U16x8 {
    uint16_t v[8];
};
struct __attribute__((aligned(16))) A16x8 {
    uint16_t v[8];
};

// 1 / (participating workers * loss scale); every worker participates without a mask.  With no
// participant at all the factor is 0, so the average comes out as zero.
__device__ inline float average_factor(int N, const int *mask, float scale, int *n_present) {
    int cnt = N;
    if (mask) {
        cnt = 0;
        for (int w = 0; w < N; ++w) cnt += mask[w] != 0;
    }
    if (n_present && blockIdx.x == 0 && threadIdx.x == 0) *n_present = cnt;
    return cnt > 0 ? 1.0f / ((float)cnt * scale) : 0.0f;
}

// 16-bit inputs: one thread owns 8 consecutive parameters and walks the workers.
template <typename T, typename Vec>
__global__ __launch_bounds__(256) void grad_average_lp_kernel(const uint16_t *g, int64_t P, int N, const float *loss_scale,
                                                              const int *mask, int *n_present, float *avg, int *found_inf) {
    const float inv = average_factor(N, mask, *loss_scale, n_present);
    const int64_t nvec = P / 8;
    bool bad = false;
    for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * blockDim.x) {
        float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int w = 0; w < N; ++w) {
            if (mask && !mask[w]) continue;
            const Vec x = *reinterpret_cast<const Vec *>(g + (int64_t)w * P + v * 8);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                bad |= Bits<T>::nonfinite(x.v[j]);
                s[j] += Bits<T>::to_f(x.v[j]);
            }
        }
        float4 o0 = make_float4(s[0] * inv, s[1] * inv, s[2] * inv, s[3] * inv);
        float4 o1 = make_float4(s[4] * inv, s[5] * inv, s[6] * inv, s[7] * inv);
        reinterpret_cast<float4 *>(avg + v * 8)[0] = o0;
        reinterpret_cast<float4 *>(avg + v * 8)[1] = o1;
    }
    // tail: fewer than 8 parameters, first block only
    if (blockIdx.x == 0) {
        const int64_t e = nvec * 8 + threadIdx.x;
        if (e < P) {
            float s = 0.0f;
            for (int w = 0; w < N; ++w) {
                if (mask && !mask[w]) continue;
                const uint16_t x = g[(int64_t)w * P + e];
                bad |= Bits<T>::nonfinite(x);
                s += Bits<T>::to_f(x);
            }
            avg[e] = s * inv;
        }
    }
    if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(found_inf, 1);
}

__global__ __launch_bounds__(256) void grad_average_f32_kernel(const float *g, int64_t P, int N, const float *loss_scale,
                                                               const int *mask, int *n_present, float *avg, int *found_inf) {
    const float inv = average_factor(N, mask, *loss_scale, n_present);
    bool bad = false;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < P; e += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int w = 0; w < N; ++w) {
            if (mask && !mask[w]) continue;
            const float x = g[(int64_t)w * P + e];
            bad |= (__float_as_uint(x) & 0x7f800000u) == 0x7f800000u;
            s += x;
        }
        avg[e] = s * inv;
    }
    if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(found_inf, 1);
}

__global__ void set_i32_kernel(int *p, int v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

struct UpdateArgs {
    int kind;
    float lr, momentum, beta1, beta2, eps, wd;
    float inv_bc1, inv_bc2;   // Adam bias corrections 1/(1-beta^step)
};

template <typename T>
__device__ inline float update_one(const UpdateArgs &u, float w, float &s1, float &s2, float g) {
    g += u.wd * w;
    if (u.kind == LSTM_OPT_SGD_MOMENTUM) {
        s1 = u.momentum * s1 - u.lr * g;       // Eq. 1
        return w + s1;                          // Eq. 2
    }
    s1 = u.beta1 * s1 + (1.0f - u.beta1) * g;
    s2 = u.beta2 * s2 + (1.0f - u.beta2) * g * g;
    const float mhat = s1 * u.inv_bc1, vhat = s2 * u.inv_bc2;
    return w - u.lr * mhat / (sqrtf(vhat) + u.eps);
}

template <typename T> struct Pack4;
template <> struct Pack4<float> {
    __device__ static inline void store(float *o, float a, float b, float c, float d) { *reinterpret_cast<float4 *>(o) = make_float4(a, b, c, d); }
};
template <> struct Pack4<_Float16> {
    __device__ static inline void store(_Float16 *o, float a, float b, float c, float d) {
        v4h v = {(_Float16)a, (_Float16)b, (_Float16)c, (_Float16)d};
        *reinterpret_cast<v4h *>(o) = v;
    }
};
template <> struct Pack4<bf16_t> {
    __device__ static inline void store(bf16_t *o, float a, float b, float c, float d) {
        uint2 v;
        v.x = Lp<bf16_t>::from_f(a).bits | ((uint32_t)Lp<bf16_t>::from_f(b).bits << 16);
        v.y = Lp<bf16_t>::from_f(c).bits | ((uint32_t)Lp<bf16_t>::from_f(d).bits << 16);
        *reinterpret_cast<uint2 *>(o) = v;
    }
};

template <typename T>
__global__ __launch_bounds__(256) void master_update_kernel(int64_t P, UpdateArgs u, float *master, float *s1, float *s2,
                                                            const float *grad, const int *found_inf, T *out) {
    if (*found_inf) return;  // overflowed step: leave every buffer untouched
    const int64_t nvec = P / 4;
    const bool adam = u.kind == LSTM_OPT_ADAM;
    for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * blockDim.x) {
        float4 w = reinterpret_cast<float4 *>(master)[v];
        float4 a = reinterpret_cast<float4 *>(s1)[v];
        float4 b = adam ? reinterpret_cast<float4 *>(s2)[v] : make_float4(0, 0, 0, 0);
        const float4 g = reinterpret_cast<const float4 *>(grad)[v];
        w.x = update_one<T>(u, w.x, a.x, b.x, g.x);
        w.y = update_one<T>(u, w.y, a.y, b.y, g.y);
        w.z = update_one<T>(u, w.z, a.z, b.z, g.z);
        w.w = update_one<T>(u, w.w, a.w, b.w, g.w);
        reinterpret_cast<float4 *>(master)[v] = w;
        reinterpret_cast<float4 *>(s1)[v] = a;
        if (adam) reinterpret_cast<float4 *>(s2)[v] = b;
        Pack4<T>::store(out + v * 4, w.x, w.y, w.z, w.w);
    }
    if (blockIdx.x == 0) {
        const int64_t e = nvec * 4 + threadIdx.x;
        if (e < P) {
            float a = s1[e], b = adam ? s2[e] : 0.0f;
            const float w = update_one<T>(u, master[e], a, b, grad[e]);
            master[e] = w;
            s1[e] = a;
            if (adam) s2[e] = b;
            out[e] = Lp<T>::from_f(w);
        }
    }
}

__global__ void scale_policy_kernel(const int *found_inf, float *loss_scale, int *good_steps, float backoff, float growth,
                                    int interval) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (*found_inf) {
        *loss_scale = *loss_scale * backoff;
        *good_steps = 0;
    } else {
        int g = *good_steps + 1;
        if (g >= interval) {
            *loss_scale = *loss_scale * growth;
            g = 0;
        }
        *good_steps = g;
    }
}

int grid_for(int64_t work_items) {
    int64_t b = (work_items + 255) / 256;
    const int64_t cap = 256 * 16;   // 16 workgroups per compute unit
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

}  // namespace
}  // namespace lstm

using namespace lstm;

namespace {
int grad_average_impl(const char *who, int64_t n_params, int32_t n_workers, const void *grads_lp, int32_t dtype,
                      const float *loss_scale, const int32_t *mask, float *avg_grad, int32_t *found_inf,
                      int32_t *n_present, void *stream) {
    if (n_params < 0 || n_workers < 1 || !loss_scale || !found_inf || (n_params > 0 && (!grads_lp || !avg_grad))) {
        set_error("%s: invalid argument (n_params=%lld n_workers=%d)", who, (long long)n_params, n_workers);
        return LSTM_ERR_INVALID;
    }
    if (dtype < LSTM_DTYPE_FP32 || dtype > LSTM_DTYPE_BF16) {
        set_error("%s: bad dtype %d", who, dtype);
        return LSTM_ERR_INVALID;
    }
    if (((uintptr_t)grads_lp | (uintptr_t)avg_grad) % 16 != 0) {
        set_error("%s: buffers must be 16-byte aligned", who);
        return LSTM_ERR_INVALID;
    }
    hipStream_t s = (hipStream_t)stream;
    // algorithmic traffic: every worker's gradient read once, the fp32 average written once
    KernelTimer timer(KC_AVERAGE, s, 0.0, (double)n_params * ((double)n_workers * dtype_size(dtype) + 4.0));
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(64), 0, s, found_inf, 0);
    LSTM_LAUNCH_CHECK();
    if (n_params == 0) return LSTM_OK;
    if (dtype == LSTM_DTYPE_FP32) {
        hipLaunchKernelGGL(grad_average_f32_kernel, dim3(grid_for(n_params)), dim3(256), 0, s, (const float *)grads_lp,
                           n_params, n_workers, loss_scale, mask, n_present, avg_grad, found_inf);
    } else {
        const uint16_t *g = (const uint16_t *)grads_lp;
        const bool aligned = (n_params % 8 == 0) || n_workers == 1;
        const int grid = grid_for(n_params / 8 + 1);
#define GA_LAUNCH(T, V)                                                                                                  \
    hipLaunchKernelGGL((grad_average_lp_kernel<T, V>), dim3(grid), dim3(256), 0, s, g, n_params, n_workers, loss_scale, \
                       mask, n_present, avg_grad, found_inf)
        if (dtype == LSTM_DTYPE_FP16) {
            if (aligned) GA_LAUNCH(_Float16, A16x8);
            else GA_LAUNCH(_Float16, U16x8);
        } else {
            if (aligned) GA_LAUNCH(bf16_t, A16x8);
            else GA_LAUNCH(bf16_t, U16x8);
        }
#undef GA_LAUNCH
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}
}  // namespace

extern "C" int grad_average(int64_t n_params, int32_t n_workers, const void *grads_lp, int32_t dtype,
                            const float *loss_scale, float *avg_grad, int32_t *found_inf, void *stream) {
    return grad_average_impl("grad_average", n_params, n_workers, grads_lp, dtype, loss_scale, nullptr, avg_grad, found_inf,
                             nullptr, stream);
}

extern "C" int grad_average_masked(int64_t n_params, int32_t n_workers, const void *grads_lp, int32_t dtype,
                                   const float *loss_scale, const int32_t *participating, float *avg_grad,
                                   int32_t *found_inf, int32_t *n_participating, void *stream) {
    if (!participating) {
        set_error("grad_average_masked: participating is NULL (use grad_average when every worker reports)");
        return LSTM_ERR_INVALID;
    }
    return grad_average_impl("grad_average_masked", n_params, n_workers, grads_lp, dtype, loss_scale, participating, avg_grad,
                             found_inf, n_participating, stream);
}

extern "C" int master_update(int64_t n_params, const optimizer_config *opt, float lr, int64_t step, float *master,
                             float *state1, float *state2, const float *avg_grad, const int32_t *found_inf,
                             float *loss_scale, int32_t *good_steps, void *params_lp_out, int32_t dtype, void *stream) {
    if (!opt || n_params < 0 || !found_inf || (n_params > 0 && (!master || !state1 || !avg_grad || !params_lp_out))) {
        set_error("master_update: null argument");
        return LSTM_ERR_INVALID;
    }
    if (opt->kind != LSTM_OPT_SGD_MOMENTUM && opt->kind != LSTM_OPT_ADAM) {
        set_error("master_update: unknown optimiser kind %d", opt->kind);
        return LSTM_ERR_INVALID;
    }
    if (opt->kind == LSTM_OPT_ADAM && (!state2 || step < 1)) {
        set_error("master_update: Adam needs state2 and step >= 1");
        return LSTM_ERR_INVALID;
    }
    if (opt->dynamic_scale && (!loss_scale || !good_steps)) {
        set_error("master_update: dynamic loss scale needs loss_scale and good_steps");
        return LSTM_ERR_INVALID;
    }
    if (dtype < LSTM_DTYPE_FP32 || dtype > LSTM_DTYPE_BF16) {
        set_error("master_update: bad dtype %d", dtype);
        return LSTM_ERR_INVALID;
    }
    if (((uintptr_t)master | (uintptr_t)state1 | (uintptr_t)state2 | (uintptr_t)avg_grad | (uintptr_t)params_lp_out) % 16 != 0) {
        set_error("master_update: buffers must be 16-byte aligned");
        return LSTM_ERR_INVALID;
    }
    hipStream_t s = (hipStream_t)stream;
    UpdateArgs u;
    u.kind = opt->kind;
    u.lr = lr;
    u.momentum = opt->momentum;
    u.beta1 = opt->beta1;
    u.beta2 = opt->beta2;
    u.eps = opt->eps;
    u.wd = opt->weight_decay;
    u.inv_bc1 = u.inv_bc2 = 1.0f;
    if (opt->kind == LSTM_OPT_ADAM) {
        u.inv_bc1 = (float)(1.0 / (1.0 - pow((double)opt->beta1, (double)step)));
        u.inv_bc2 = (float)(1.0 / (1.0 - pow((double)opt->beta2, (double)step)));
    }
    // algorithmic traffic per parameter: read master, state(s), gradient; write master, state(s), working copy
    // SGD: 3 reads + 2 writes of fp32 (20 B) + the working copy; Adam: 4 reads + 3 writes (28 B) + the working copy
    const double per_param = (opt->kind == LSTM_OPT_ADAM ? 7.0 : 5.0) * 4.0 + (double)dtype_size(dtype);
    KernelTimer timer(KC_UPDATE, s, 0.0, (double)n_params * per_param);
    if (n_params > 0) {
        const int grid = grid_for(n_params / 4 + 1);
        switch (dtype) {
            case LSTM_DTYPE_FP32:
                hipLaunchKernelGGL(master_update_kernel<float>, dim3(grid), dim3(256), 0, s, n_params, u, master, state1, state2, avg_grad, found_inf, (float *)params_lp_out);
                break;
            case LSTM_DTYPE_FP16:
                hipLaunchKernelGGL(master_update_kernel<_Float16>, dim3(grid), dim3(256), 0, s, n_params, u, master, state1, state2, avg_grad, found_inf, (_Float16 *)params_lp_out);
                break;
            default:
                hipLaunchKernelGGL(master_update_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, n_params, u, master, state1, state2, avg_grad, found_inf, (bf16_t *)params_lp_out);
        }
        LSTM_LAUNCH_CHECK();
    }
    if (opt->dynamic_scale) {
        hipLaunchKernelGGL(scale_policy_kernel, dim3(1), dim3(64), 0, s, found_inf, loss_scale, good_steps, opt->scale_backoff,
                           opt->scale_growth, opt->growth_interval);
        LSTM_LAUNCH_CHECK();
    }
    return LSTM_OK;
}

extern "C" float lr_schedule(float lr0, int32_t n_workers, float n_half, float eff_lr_max, int32_t warmup_steps, float gamma,
                             int64_t index) {
    if (n_workers < 1 || !(n_half > 0.0f) || index < 0) return 0.0f;
    double base = (double)lr0 / (1.0 + (double)n_workers / (double)n_half);          // Eq. 4
    if (base * n_workers > (double)eff_lr_max) base = (double)eff_lr_max / n_workers;  // clip of the effective rate
    if (warmup_steps > 0 && index < warmup_steps) return (float)(base * (double)(index + 1) / (double)warmup_steps);
    const double e = warmup_steps > 0 ? (double)(index - warmup_steps + 1) : (double)index;
    return (float)(base * pow((double)gamma, e));                                     // Eq. 3
}
