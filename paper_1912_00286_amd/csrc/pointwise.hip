// Pointwise, layout and small reduction kernels of the LSTM training step:
// gate non-linearities forward/backward, transposes, column sums, the output
// head with its loss, embedding gather / scatter-add, casts and fills.
#include "kernels.h"
#include "packed.h"

namespace lstm {

#define LSTM_DISPATCH(dtype, T, ...)                               \
    switch (dtype) {                                               \
        case LSTM_DTYPE_FP32: { using T = float; __VA_ARGS__; } break;    \
        case LSTM_DTYPE_FP16: { using T = _Float16; __VA_ARGS__; } break; \
        case LSTM_DTYPE_BF16: { using T = bf16_t; __VA_ARGS__; } break;   \
        default: set_error("bad dtype %d", dtype); return LSTM_ERR_INVALID; \
    }

// 16-bit storage types only (the 16-byte vector kernels)
#define LP16_DISPATCH(dtype, T, ...)                               \
    switch (dtype) {                                               \
        case LSTM_DTYPE_FP16: { using T = _Float16; __VA_ARGS__; } break; \
        case LSTM_DTYPE_BF16: { using T = bf16_t; __VA_ARGS__; } break;   \
        default: set_error("bad dtype %d", dtype); return LSTM_ERR_INVALID; \
    }

namespace {

// Rows of several simulated workers interleave in the time-major activations: logical row r of
// worker w (its own [T, seg] rows) lies at (r / seg) * (workers * seg) + w * seg + r % seg.
// One worker: the identity.
struct RowSeg {
    int workers, seg;
    __device__ inline int64_t row(int r, int w) const { return (int64_t)(r / seg) * workers * seg + (int64_t)w * seg + r % seg; }
};

// The fp32 baseline mode uses the accurate library functions; the
// low-precision modes use the hardware exponential.
template <typename T> struct Act {
    __device__ static inline float sigmoid(float a) { return sigmoidf_dev(a); }
    __device__ static inline float tanh(float a) { return tanhf_dev(a); }
};
template <> struct Act<float> {
    __device__ static inline float sigmoid(float a) { return 1.0f / (1.0f + expf(-a)); }
    __device__ static inline float tanh(float a) { return tanhf(a); }
};

inline int blocks_for(int64_t n, int threads, int cap = 65535 * 16) {
    int64_t b = (n + threads - 1) / threads;
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

__global__ void fill_u32_kernel(uint32_t *dst, uint32_t v, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) dst[i] = v;
}

template <typename T>
__global__ void init_state_kernel(const T *h0, const float *c0, T *h_slot0, T *c_slot0, float *c_state, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        h_slot0[i] = h0 ? h0[i] : Lp<T>::from_f(0.0f);
        const float c = c0 ? c0[i] : 0.0f;
        c_slot0[i] = Lp<T>::from_f(c);
        c_state[i] = c;
    }
}

template <typename T>
__global__ void gates_forward_kernel(const float *A, float *c_state, T *gates, T *c_out, T *h_out, int B, int H) {
    const int64_t n = (int64_t)B * H;
    const int G = 4 * H;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(e / H), j = (int)(e % H);
        const float *a = A + (int64_t)b * G;
        const float i = Act<T>::sigmoid(a[j]);
        const float f = Act<T>::sigmoid(a[H + j]);
        const float g = Act<T>::tanh(a[2 * H + j]);
        const float o = Act<T>::sigmoid(a[3 * H + j]);
        const float c = f * c_state[e] + i * g;
        const float h = o * Act<T>::tanh(c);
        c_state[e] = c;
        T *gr = gates + (int64_t)b * G;
        gr[j] = Lp<T>::from_f(i);
        gr[H + j] = Lp<T>::from_f(f);
        gr[2 * H + j] = Lp<T>::from_f(g);
        gr[3 * H + j] = Lp<T>::from_f(o);
        c_out[e] = Lp<T>::from_f(c);
        h_out[e] = Lp<T>::from_f(h);
    }
}

template <typename T>
__global__ void gates_backward_kernel(const T *dh_above, const float *dh_rec, const T *gates, const T *c_t,
                                      const T *c_prev, float *dc_state, T *dA, int B, int H, int first, int n_rec) {
    const int64_t n = (int64_t)B * H;
    const int G = 4 * H;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int b = (int)(e / H), j = (int)(e % H);
        const T *gr = gates + (int64_t)b * G;
        const float i = Lp<T>::to_f(gr[j]), f = Lp<T>::to_f(gr[H + j]);
        const float g = Lp<T>::to_f(gr[2 * H + j]), o = Lp<T>::to_f(gr[3 * H + j]);
        const float tc = Act<T>::tanh(Lp<T>::to_f(c_t[e]));
        float dh = dh_above ? Lp<T>::to_f(dh_above[e]) : 0.0f;
        if (dh_rec)
            for (int q = 0; q < n_rec; ++q) dh += dh_rec[(int64_t)q * n + e];
        const float dcr = first ? 0.0f : dc_state[e];
        const float d_o = dh * tc;
        const float dc = dcr + dh * o * (1.0f - tc * tc);
        const float di = dc * g, dg = dc * i, df = dc * Lp<T>::to_f(c_prev[e]);
        dc_state[e] = dc * f;
        T *da = dA + (int64_t)b * G;
        da[j] = Lp<T>::from_f(di * i * (1.0f - i));
        da[H + j] = Lp<T>::from_f(df * f * (1.0f - f));
        da[2 * H + j] = Lp<T>::from_f(dg * (1.0f - g * g));
        da[3 * H + j] = Lp<T>::from_f(d_o * o * (1.0f - o));
    }
}

// 64x64 tile transpose through LDS; 256 threads
template <typename U>
__global__ __launch_bounds__(256) void transpose_kernel(const U *in, int64_t ld_in, U *out, int64_t ld_out, int R, int C) {
    __shared__ U tile[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int rr = ty; rr < 64; rr += 4) {
        const int r = r0 + rr, c = c0 + tx;
        if (r < R && c < C) tile[rr][tx] = in[(int64_t)r * ld_in + c];
    }
    __syncthreads();
    for (int cc = ty; cc < 64; cc += 4) {
        const int c = c0 + cc, r = r0 + tx;
        if (r < R && c < C) out[(int64_t)c * ld_out + r] = tile[tx][cc];
    }
}

constexpr int CS_ROWS = 512;  // rows per column-sum chunk
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *in, int64_t ld, int R, int C, const float *row_w,
                                                             float *partial, RowSeg rs) {
    __shared__ float red[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63);
    const int ry = threadIdx.x >> 6;
    const int r_beg = blockIdx.y * CS_ROWS, r_end = min(R, r_beg + CS_ROWS);
    float s = 0.0f;
    if (c < C)
        for (int r = r_beg + ry; r < r_end; r += 4) {
            const int64_t pr = rs.row(r, blockIdx.z);
            const float v = Lp<T>::to_f(in[pr * ld + c]);
            s += row_w ? row_w[pr] * v : v;
        }
    red[ry][threadIdx.x & 63] = s;
    __syncthreads();
    if (ry == 0 && c < C)
        partial[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * C + c] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}
// 16-bit types, 8 columns (one 16-byte load) per thread: a wavefront reads 1 KB of a row at once
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_vec_kernel(const T *in, int64_t ld, int R, int C, const float *row_w,
                                                                 float *partial, RowSeg rs) {
    __shared__ float red[4][64][9];
    const int lane = threadIdx.x & 63, ry = threadIdx.x >> 6;
    const int c = blockIdx.x * 512 + lane * 8;
    const int r_beg = blockIdx.y * CS_ROWS, r_end = min(R, r_beg + CS_ROWS);
    float s[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    if (c < C)
#pragma unroll 8
        for (int r = r_beg + ry; r < r_end; r += 4) {
            const int64_t pr = rs.row(r, blockIdx.z);
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(in + pr * ld + c);
            T v[8];
            __builtin_memcpy(v, &raw, 16);
            const float w = row_w ? row_w[pr] : 1.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += row_w ? w * Lp<T>::to_f(v[e]) : Lp<T>::to_f(v[e]);
        }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[ry][lane][e] = s[e];
    __syncthreads();
    for (int i = threadIdx.x; i < 512; i += 256) {
        const int l = i >> 3, e = i & 7;
        if ((int)blockIdx.x * 512 + i < C)
            partial[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * C + blockIdx.x * 512 + i] =
                (red[0][l][e] + red[1][l][e]) + (red[2][l][e] + red[3][l][e]);
    }
}
// Column sums of a tensor stored in 64x64 blocks ([row block][ncb][64][64], zero padded): a
// workgroup owns one column block and up to CSB_BLOCKS row blocks, reads them as whole 8 KB
// blocks (thread = 8 columns of one of 32 row slots) and writes one partial row.
constexpr int CSB_BLOCKS = 8;
// packed: every block is in MFMA-fragment order instead (16 bytes = 8 columns of one row, the rows of a 32-row half one
// after the other); the threads then take consecutive rows, so that a wavefront still reads whole lines.
template <typename T>
__global__ __launch_bounds__(256) void colsum_blocked_partial_kernel(const T *blk, int ncb, int nrb, int C, float *partial, int seg,
                                                                     int stride, int packed) {
    // Several workers (blockIdx.z): worker z owns `seg` consecutive row blocks out of every `stride`
    // (its rows of one time step); its i-th row block is (i / seg) * stride + z * seg + i % seg.
    // One worker: seg = stride, which makes that i.
    __shared__ float red[32][65];
    const int cb = blockIdx.x;
    const int c8 = (packed ? threadIdx.x >> 5 : threadIdx.x & 7) * 8, rs = packed ? threadIdx.x & 31 : threadIdx.x >> 3;
    const int rb0 = blockIdx.y * CSB_BLOCKS, rb1 = min(nrb, rb0 + CSB_BLOCKS);
    float s[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int i = rb0; i < rb1; ++i) {
        const int64_t rb = (int64_t)(i / seg) * stride + (int64_t)blockIdx.z * seg + i % seg;
        const T *b = blk + (rb * ncb + cb) * 4096;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(b + (packed ? frag_offset(rs + 32 * h, c8, 2) : (rs + 32 * h) * 64 + c8));
            T v[8];
            __builtin_memcpy(v, &raw, 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] += Lp<T>::to_f(v[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rs][c8 + e] = s[e];
    __syncthreads();
    if (threadIdx.x < 64) {
        float t = 0.0f;
#pragma unroll
        for (int r = 0; r < 32; ++r) t += red[r][threadIdx.x];
        const int c = cb * 64 + threadIdx.x;
        if (c < C) partial[((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * C + c] = t;
    }
}
// (one-wavefront workgroups: a thread adds up a whole column of partial sums, so the columns should spread over as
// many compute units as possible)
template <typename T>
__global__ void colsum_final_kernel(const float *partial, int chunks, int C, const float *scale_dev, T *out, int64_t out_stride) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    // four running sums, so that the loads of consecutive chunks do not wait for each other's additions
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    const float *p = partial + (int64_t)blockIdx.y * chunks * C + c;
    int k = 0;
    for (; k + 4 <= chunks; k += 4) {
        s0 += p[(int64_t)k * C]; s1 += p[(int64_t)(k + 1) * C]; s2 += p[(int64_t)(k + 2) * C]; s3 += p[(int64_t)(k + 3) * C];
    }
    for (; k < chunks; ++k) s0 += p[(int64_t)k * C];
    float s = (s0 + s1) + (s2 + s3);
    if (scale_dev) s *= *scale_dev;
    out[blockIdx.y * out_stride + c] = Lp<T>::from_f(s);
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// one wavefront per output row; 4 rows per workgroup
template <typename T>
__global__ __launch_bounds__(256) void head_forward_kernel(int head, const T *h_top, const T *w, const T *b,
                                                           const float *targets, int rows, int H, float inv_M,
                                                           float *dzu, float *partial) {
    __shared__ float wl[4];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wv;
    float ell = 0.0f;
    if (row < rows) {
        const T *hr = h_top + (int64_t)row * H;
        float s = 0.0f;
        for (int j = lane; j < H; j += 64) s += Lp<T>::to_f(hr[j]) * Lp<T>::to_f(w[j]);
        s = wave_sum(s);
        if (lane == 0) {
            const float z = s + Lp<T>::to_f(b[0]);
            const float y = targets[row];
            float d;
            if (head == LSTM_HEAD_STEP_MSE) {
                const float r = z - y;
                ell = r * r;
                d = 2.0f * r;
            } else if (head == LSTM_HEAD_FC_HINGE) {
                const float m = 1.0f - y * z;            // Eq. 6 without the multiplier; labels +-1
                ell = fmaxf(m, 0.0f);
                d = m > 0.0f ? -y : 0.0f;
            } else {
                const float az = fabsf(z);
                const float e = expf(-az);
                ell = fmaxf(z, 0.0f) - z * y + log1pf(e);
                const float sg = z >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
                d = sg - y;
            }
            dzu[row] = d * inv_M;
        }
    }
    if (lane == 0) wl[wv] = ell;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (wl[0] + wl[1]) + (wl[2] + wl[3]);
}
// The same with 16-byte loads (H % 8 == 0, aligned rows): LPR lanes (a power of two, at most 64) share a
// row, each lane-group takes the four consecutive rows of one partial sum.
template <typename T>
__device__ __forceinline__ float dot8(const u32x4 &a, const u32x4 &b) {
    __attribute__((aligned(16))) T x[8], y[8];
    *reinterpret_cast<u32x4 *>(x) = a;
    *reinterpret_cast<u32x4 *>(y) = b;
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) s += Lp<T>::to_f(x[k]) * Lp<T>::to_f(y[k]);
    return s;
}
template <typename T>
__global__ __launch_bounds__(256) void head_forward_vec_kernel(int head, const T *h_top, const T *w, const T *b,
                                                               const float *targets, int rows, int H, float inv_M,
                                                               float *dzu, float *partial, int lpr) {
    const int nvec = H / 8;
    const int sub = threadIdx.x & (lpr - 1);
    const int64_t group = ((int64_t)blockIdx.x * 256 + threadIdx.x) / lpr;      // rows 4 group .. 4 group + 3
    const int64_t row0 = group * 4;
    if (row0 >= rows) return;                          // whole lane-groups leave together; no barrier below
    const u32x4 *wv = reinterpret_cast<const u32x4 *>(w);
    float dot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int v = sub; v < nvec; v += lpr) {
        const u32x4 wq = wv[v];
        u32x4 hq[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t r = row0 + k < rows ? row0 + k : rows - 1;
            hq[k] = reinterpret_cast<const u32x4 *>(h_top + r * H)[v];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) dot[k] += dot8<T>(hq[k], wq);
    }
    for (int off = lpr >> 1; off > 0; off >>= 1) {
#pragma unroll
        for (int k = 0; k < 4; ++k) dot[k] += __shfl_xor(dot[k], off, 64);
    }
    if (sub != 0) return;
    const float bias = Lp<T>::to_f(b[0]);
    float ell_sum = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (row0 + k >= rows) break;
        const float z = dot[k] + bias;
        const float y = targets[row0 + k];
        float d, ell;
        if (head == LSTM_HEAD_STEP_MSE) {
            const float r = z - y;
            ell = r * r;
            d = 2.0f * r;
        } else if (head == LSTM_HEAD_FC_HINGE) {
            const float m = 1.0f - y * z;
            ell = fmaxf(m, 0.0f);
            d = m > 0.0f ? -y : 0.0f;
        } else {
            const float az = fabsf(z);
            const float e = expf(-az);
            ell = fmaxf(z, 0.0f) - z * y + log1pf(e);
            const float sg = z >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
            d = sg - y;
        }
        dzu[row0 + k] = d * inv_M;
        ell_sum += ell;
    }
    partial[group] = ell_sum;
}
// one workgroup per worker: partial sum i covers rows 4i..4i+3, all of one worker (seg % 4 == 0
// whenever there are several)
__global__ __launch_bounds__(256) void loss_final_kernel(const float *partial, int n, float inv_M, float *loss, RowSeg rs) {
    __shared__ double red[256];
    double s = 0.0;
    if (rs.workers == 1) {
        for (int i = threadIdx.x; i < n; i += 256) s += (double)partial[i];
    } else {
        // this worker's rows are seg consecutive rows of every time step: seg / 4 consecutive partial sums per step
        const int per_step = rs.seg / 4, stride = rs.workers * per_step, steps = n / stride;
        for (int k = threadIdx.x; k < steps * per_step; k += 256)
            s += (double)partial[(int64_t)(k / per_step) * stride + (int)blockIdx.x * per_step + k % per_step];
    }
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[blockIdx.x] = (float)(red[0] * (double)inv_M);
}

// relu_of: when given, the output is the derivative through a ReLU whose result relu_of holds
// (zero wherever that result is zero)
template <typename T>
__global__ void head_backward_dh_kernel(const float *dzu, const T *w, const float *scale_dev, const T *relu_of, T *dh,
                                        int rows, int H) {
    const float S = *scale_dev;
    const int64_t n = (int64_t)rows * H;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / H), j = (int)(e % H);
        float v = S * dzu[r] * Lp<T>::to_f(w[j]);
        if (relu_of && !(Lp<T>::to_f(relu_of[e]) > 0.0f)) v = 0.0f;
        dh[e] = Lp<T>::from_f(v);
    }
}
template <typename T>
__global__ void head_backward_dh_vec_kernel(const float *dzu, const T *w, const float *scale_dev, const T *relu_of, T *dh,
                                            int rows, int H) {
    const float S = *scale_dev;
    const int nvec = H / 8;
    const int64_t n = (int64_t)rows * nvec;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / nvec), v = (int)(e % nvec);
        __attribute__((aligned(16))) T wq[8], rq[8], out[8];
        *reinterpret_cast<u32x4 *>(wq) = reinterpret_cast<const u32x4 *>(w)[v];
        if (relu_of) *reinterpret_cast<u32x4 *>(rq) = reinterpret_cast<const u32x4 *>(relu_of)[e];
        const float g = S * dzu[r];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float x = g * Lp<T>::to_f(wq[k]);
            if (relu_of && !(Lp<T>::to_f(rq[k]) > 0.0f)) x = 0.0f;
            out[k] = Lp<T>::from_f(x);
        }
        reinterpret_cast<u32x4 *>(dh)[e] = *reinterpret_cast<const u32x4 *>(out);
    }
}
template <typename T>
__global__ void relu_inplace_kernel(T *a, int64_t n) {
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const float v = Lp<T>::to_f(a[e]);
        if (!(v > 0.0f)) a[e] = Lp<T>::from_f(0.0f);
    }
}
template <typename T>
__global__ __launch_bounds__(256) void head_backward_bias_kernel(const float *dzu, const float *scale_dev, int rows, T *out,
                                                                 RowSeg rs, int64_t out_stride) {
    __shared__ double red[256];
    double s = 0.0;
#pragma unroll 8
    for (int i = threadIdx.x; i < rows; i += 256) s += (double)dzu[rs.row(i, blockIdx.x)];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x * out_stride] = Lp<T>::from_f((float)(red[0] * (double)(*scale_dev)));
}

template <typename T>
__global__ void embed_gather_kernel(const int32_t *ids, const T *E, T *X, int rows, int V, int D) {
    const int64_t n = (int64_t)rows * D;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
        const int r = (int)(e / D), d = (int)(e % D);
        int id = ids[r];
        id = id < 0 ? 0 : (id >= V ? V - 1 : id);
        X[e] = E[(int64_t)id * D + d];
    }
}
// dE[id[r]] += dX[r].  Token frequencies are heavy-tailed (a bounded Zipf law here), so plain atomics
// serialise on the few hottest rows of the table: thousands of additions to the same 128 addresses.  Each
// workgroup therefore owns a contiguous slice of the tokens, sums the rows with id < hot_rows in LDS and
// adds that table to memory once at the end; all other rows go to memory directly.  Correct for any ids
// (the split is by value, not by frequency); the summation order is not fixed either way.
constexpr int SCATTER_LDS_FLOATS = 8192;
template <typename T>
__global__ __launch_bounds__(256) void embed_scatter_kernel(const int32_t *ids, const T *dX, float *dE, int rows, int V, int D,
                                                            int rows_per_wg, int hot_rows) {
    __shared__ float hot[SCATTER_LDS_FLOATS];
    const int hot_n = hot_rows * D;
    for (int i = threadIdx.x; i < hot_n; i += 256) hot[i] = 0.0f;
    __syncthreads();
    const int r0 = blockIdx.x * rows_per_wg, r1 = min(rows, r0 + rows_per_wg);
    for (int64_t e = (int64_t)r0 * D + threadIdx.x; e < (int64_t)r1 * D; e += 256) {
        const int r = (int)(e / D), d = (int)(e % D);
        int id = ids[r];
        id = id < 0 ? 0 : (id >= V ? V - 1 : id);
        const float v = Lp<T>::to_f(dX[e]);
        if (id < hot_rows) atomicAdd(&hot[id * D + d], v);
        else atomicAdd(&dE[(int64_t)id * D + d], v);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < hot_n; i += 256) {
        const float v = hot[i];
        if (v != 0.0f) atomicAdd(&dE[i], v);
    }
}
template <typename T>
__global__ void cast_kernel(const float *in, T *out, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) out[i] = Lp<T>::from_f(in[i]);
}
template <typename T>
__global__ void copy_state_kernel(const T *h_src, const float *c_src, T *h_dst, float *c_dst, int64_t n) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        if (h_dst) h_dst[i] = h_src[i];
        if (c_dst) c_dst[i] = c_src[i];
    }
}

}  // namespace

int fill_u32(void *dst, uint32_t value, int64_t n_words, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (n_words <= 0) return LSTM_OK;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n_words, 256, 8192)), dim3(256), 0, s, (uint32_t *)dst, value, n_words);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int init_state(int dtype, const void *h0, const float *c0, void *h_slot0, void *c_slot0, float *c_state, int64_t n,
               hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(init_state_kernel<T>, dim3(blocks_for(n, 256, 4096)), dim3(256), 0, s,
                                               (const T *)h0, c0, (T *)h_slot0, (T *)c_slot0, c_state, n));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int gates_forward(int dtype, const float *A, float *c_state, void *gates, void *c_out, void *h_out, int B, int H,
                  hipStream_t s) {
    KernelTimer timer(KC_POINTWISE, s, 0.0, (double)B * H * (16.0 + 4.0 + 4.0 + 6.0 * sizeof(uint16_t)));
    const int64_t n = (int64_t)B * H;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(gates_forward_kernel<T>, dim3(blocks_for(n, 256, 8192)), dim3(256), 0, s, A,
                                               c_state, (T *)gates, (T *)c_out, (T *)h_out, B, H));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int gates_backward(int dtype, const void *dh_above, const float *dh_rec, const void *gates, const void *c_t,
                   const void *c_prev, float *dc_state, void *dA, int B, int H, int first, int n_rec, hipStream_t s) {
    KernelTimer timer(KC_POINTWISE, s, 0.0, (double)B * H * (8.0 + 4.0 + 11.0 * sizeof(uint16_t)));
    const int64_t n = (int64_t)B * H;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(gates_backward_kernel<T>, dim3(blocks_for(n, 256, 8192)), dim3(256), 0, s,
                                               (const T *)dh_above, dh_rec, (const T *)gates, (const T *)c_t,
                                               (const T *)c_prev, dc_state, (T *)dA, B, H, first, n_rec));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int transpose_lp(int dtype, const void *in, int64_t ld_in, void *out, int64_t ld_out, int R, int C, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (R <= 0 || C <= 0) return LSTM_OK;
    dim3 grid((C + 63) / 64, (R + 63) / 64);
    if (grid.y > 65535u) {
        set_error("transpose: too many rows %d", R);
        return LSTM_ERR_UNSUPPORTED;
    }
    if (dtype == LSTM_DTYPE_FP32)
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s, (const uint32_t *)in, ld_in, (uint32_t *)out, ld_out, R, C);
    else
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)in, ld_in, (uint16_t *)out, ld_out, R, C);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int colsum_chunks(int R) { return R <= 0 ? 1 : (R + CS_ROWS - 1) / CS_ROWS; }

int colsum(int dtype, const void *in, int64_t ld, int R, int C, const float *row_w, const float *scale_dev,
           float *partial, void *out_lp, hipStream_t s, int workers, int seg, int64_t out_stride) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (C <= 0) return LSTM_OK;
    const int chunks = colsum_chunks(R);
    const RowSeg rs{workers, workers > 1 ? seg : (R > 0 ? R : 1)};
    dim3 grid((C + 63) / 64, chunks, workers);
    if (grid.y > 65535u || workers > 65535 || workers < 1 || rs.seg < 1) {
        set_error("colsum: too many rows %d", R);
        return LSTM_ERR_UNSUPPORTED;
    }
    const bool vec = dtype != LSTM_DTYPE_FP32 && C % 8 == 0 && ld % 8 == 0 && (uintptr_t)in % 16 == 0;
    LSTM_DISPATCH(dtype, T, {
        if constexpr (sizeof(T) == 2) {
            if (vec)
                hipLaunchKernelGGL(colsum_partial_vec_kernel<T>, dim3((C + 511) / 512, chunks, workers), dim3(256), 0, s,
                                   (const T *)in, ld, R, C, row_w, partial, rs);
        }
        if (!vec) hipLaunchKernelGGL(colsum_partial_kernel<T>, grid, dim3(256), 0, s, (const T *)in, ld, R, C, row_w, partial, rs);
        hipLaunchKernelGGL(colsum_final_kernel<T>, dim3((C + 63) / 64, workers), dim3(64), 0, s, partial, chunks, C, scale_dev,
                           (T *)out_lp, out_stride);
    });
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int colsum_blocked_chunks(int R) { return R <= 0 ? 1 : ((R + 63) / 64 + CSB_BLOCKS - 1) / CSB_BLOCKS; }

int colsum_blocked(int dtype, const void *blk, int ncb, int R, int C, float *partial, void *out_lp, hipStream_t s, int workers,
                   int seg_rows, int64_t out_stride, int packed) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (C <= 0) return LSTM_OK;
    // R rows per worker; with several workers every time step holds `workers` segments of seg_rows rows
    const int nrb = (R + 63) / 64, chunks = colsum_blocked_chunks(R);
    if (dtype == LSTM_DTYPE_FP32 || chunks > 65535 || (C + 63) / 64 > ncb || workers < 1 || workers > 65535 ||
        (workers > 1 && (seg_rows < 64 || seg_rows % 64 != 0 || R % seg_rows != 0))) {
        set_error("colsum_blocked: unsupported (dtype %d, R=%d, C=%d, ncb=%d, workers=%d, segment %d)", dtype, R, C, ncb, workers,
                  seg_rows);
        return LSTM_ERR_UNSUPPORTED;
    }
    const int seg = workers > 1 ? seg_rows / 64 : (nrb > 0 ? nrb : 1), stride = seg * workers;
    LSTM_DISPATCH(dtype, T, {
        if constexpr (sizeof(T) == 2)
            hipLaunchKernelGGL(colsum_blocked_partial_kernel<T>, dim3((C + 63) / 64, chunks, workers), dim3(256), 0, s, (const T *)blk,
                               ncb, nrb, C, partial, seg, stride, packed);
        hipLaunchKernelGGL(colsum_final_kernel<T>, dim3((C + 63) / 64, workers), dim3(64), 0, s, partial, chunks, C,
                           (const float *)nullptr, (T *)out_lp, out_stride);
    });
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int colsum_finish(int dtype, const float *partial, int chunks, int C, void *out_lp, hipStream_t s, int workers, int64_t out_stride) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (C <= 0) return LSTM_OK;
    if (dtype == LSTM_DTYPE_FP32 || chunks < 1 || workers < 1 || workers > 65535 || !partial || !out_lp) {
        set_error("colsum_finish: unsupported (dtype %d, %d chunks, %d workers)", dtype, chunks, workers);
        return LSTM_ERR_UNSUPPORTED;
    }
    LSTM_DISPATCH(dtype, T, {
        hipLaunchKernelGGL(colsum_final_kernel<T>, dim3((C + 63) / 64, workers), dim3(64), 0, s, partial, chunks, C,
                           (const float *)nullptr, (T *)out_lp, out_stride);
    });
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int head_loss_blocks(int rows) { return rows <= 0 ? 1 : (rows + 3) / 4; }

int head_forward(int dtype, int head, const void *h_top, const void *w, const void *b, const float *targets, int rows,
                 int H, int M_total, float *dzu, float *partial, float *loss, hipStream_t s, int workers, int seg) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    const int nb = head_loss_blocks(rows);
    const float inv_M = 1.0f / (float)M_total;
    const RowSeg rs{workers, workers > 1 ? seg : 1};
    const bool vec = dtype != LSTM_DTYPE_FP32 && H % 8 == 0 && ((uintptr_t)h_top | (uintptr_t)w) % 16 == 0;
    if (vec) {
        int lpr = 1;
        while (lpr < 64 && lpr < H / 8) lpr <<= 1;
        const int groups_per_wg = 256 / lpr;
        LP16_DISPATCH(dtype, T, hipLaunchKernelGGL(head_forward_vec_kernel<T>, dim3((nb + groups_per_wg - 1) / groups_per_wg), dim3(256),
                                                   0, s, head, (const T *)h_top, (const T *)w, (const T *)b, targets, rows, H, inv_M,
                                                   dzu, partial, lpr));
    } else {
        LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(head_forward_kernel<T>, dim3(nb), dim3(256), 0, s, head, (const T *)h_top,
                                                   (const T *)w, (const T *)b, targets, rows, H, inv_M, dzu, partial));
    }
    LSTM_LAUNCH_CHECK();
    hipLaunchKernelGGL(loss_final_kernel, dim3(workers), dim3(256), 0, s, partial, nb, inv_M, loss, rs);
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int head_backward_dh(int dtype, const float *dzu, const void *w, const float *scale_dev, const void *relu_of, void *dh,
                     int rows, int H, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    const int64_t n = (int64_t)rows * H;
    const bool vec = dtype != LSTM_DTYPE_FP32 && H % 8 == 0 && ((uintptr_t)w | (uintptr_t)relu_of | (uintptr_t)dh) % 16 == 0;
    if (vec) {
        LP16_DISPATCH(dtype, T, hipLaunchKernelGGL(head_backward_dh_vec_kernel<T>, dim3(blocks_for(n / 8, 256, 8192)), dim3(256), 0, s,
                                                   dzu, (const T *)w, scale_dev, (const T *)relu_of, (T *)dh, rows, H));
    } else {
        LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(head_backward_dh_kernel<T>, dim3(blocks_for(n, 256, 8192)), dim3(256), 0, s,
                                                   dzu, (const T *)w, scale_dev, (const T *)relu_of, (T *)dh, rows, H));
    }
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int relu_inplace(int dtype, void *a, int64_t n, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (n <= 0) return LSTM_OK;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(relu_inplace_kernel<T>, dim3(blocks_for(n, 256, 8192)), dim3(256), 0, s, (T *)a, n));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int head_backward_bias(int dtype, const float *dzu, const float *scale_dev, int rows, void *out_lp, hipStream_t s, int workers,
                       int seg, int64_t out_stride) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    const RowSeg rs{workers, workers > 1 ? seg : (rows > 0 ? rows : 1)};
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(head_backward_bias_kernel<T>, dim3(workers), dim3(256), 0, s, dzu, scale_dev, rows,
                                               (T *)out_lp, rs, out_stride));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int embed_gather(int dtype, const int32_t *ids, const void *E, void *X, int rows, int V, int D, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    const int64_t n = (int64_t)rows * D;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(embed_gather_kernel<T>, dim3(blocks_for(n, 256, 16384)), dim3(256), 0, s, ids,
                                               (const T *)E, (T *)X, rows, V, D));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int embed_scatter_add(int dtype, const int32_t *ids, const void *dX, float *dE32, int rows, int V, int D, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (rows <= 0 || D <= 0) return LSTM_OK;
    int hot_rows = SCATTER_LDS_FLOATS / D;                     // rows of the table summed in LDS (0: D too wide, all direct)
    if (hot_rows > 64) hot_rows = 64;
    if (hot_rows > V) hot_rows = V;
    // about two workgroups per four compute units: few enough that the hot rows see little contention
    int rows_per_wg = (rows + 127) / 128;
    if (rows_per_wg < 16) rows_per_wg = 16;
    const int grid = (rows + rows_per_wg - 1) / rows_per_wg;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(embed_scatter_kernel<T>, dim3(grid), dim3(256), 0, s, ids, (const T *)dX, dE32, rows, V,
                                               D, rows_per_wg, hot_rows));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int cast_f32_to_lp(int dtype, const float *in, void *out, int64_t n, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (n <= 0) return LSTM_OK;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(cast_kernel<T>, dim3(blocks_for(n, 256, 16384)), dim3(256), 0, s, in, (T *)out, n));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

int copy_state(int dtype, const void *h_src, const float *c_src, void *h_dst, float *c_dst, int64_t n, hipStream_t s) {
    KernelTimer timer(KC_AUX, s, 0.0, 0.0);
    if (!h_dst && !c_dst) return LSTM_OK;
    LSTM_DISPATCH(dtype, T, hipLaunchKernelGGL(copy_state_kernel<T>, dim3(blocks_for(n, 256, 4096)), dim3(256), 0, s,
                                               (const T *)h_src, c_src, (T *)h_dst, c_dst, n));
    LSTM_LAUNCH_CHECK();
    return LSTM_OK;
}

}  // namespace lstm
