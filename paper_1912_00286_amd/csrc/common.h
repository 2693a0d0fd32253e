// Shared declarations of the gfx950 LSTM training-step library (internal).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lstm_mi355.h"
#include "../../include/lstm_mi355_debug.h"

namespace lstm {

// ---------------------------------------------------------------- error plumbing
void set_error(const char *fmt, ...);

#define LSTM_HIP_TRY(expr)                                                                  \
    do {                                                                                    \
        hipError_t _e = (expr);                                                             \
        if (_e != hipSuccess) {                                                             \
            ::lstm::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
            return LSTM_ERR_HIP;                                                            \
        }                                                                                   \
    } while (0)

#define LSTM_TRY(expr)                  \
    do {                                \
        int _s = (expr);                \
        if (_s != LSTM_OK) return _s;   \
    } while (0)

#define LSTM_LAUNCH_CHECK() LSTM_HIP_TRY(hipGetLastError())

// ---------------------------------------------------------------- storage types
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef __bf16 v8b __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
// 16 bytes of packed 16-bit elements as a native vector (HIP's uint4 is a struct
// wrapping a union, which keeps register arrays of it from being scalarised)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct bf16_t {
    uint16_t bits;
};

__host__ __device__ inline float bf16_to_float(bf16_t v) {
    union { uint32_t u; float f; } c;
    c.u = ((uint32_t)v.bits) << 16;
    return c.f;
}
// round to nearest even; NaN stays NaN
__host__ __device__ inline bf16_t float_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    bf16_t r;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) {
        r.bits = (uint16_t)((c.u >> 16) | 0x40u);
    } else {
        c.u += 0x7fffu + ((c.u >> 16) & 1u);
        r.bits = (uint16_t)(c.u >> 16);
    }
    return r;
}

template <typename T> struct Lp;
template <> struct Lp<float> {
    static constexpr int code = LSTM_DTYPE_FP32;
    __device__ static inline float to_f(float v) { return v; }
    __device__ static inline float from_f(float v) { return v; }
};
template <> struct Lp<_Float16> {
    static constexpr int code = LSTM_DTYPE_FP16;
    __device__ static inline float to_f(_Float16 v) { return (float)v; }
    __device__ static inline _Float16 from_f(float v) { return (_Float16)v; }  // RNE, overflow -> inf
    __device__ static inline v16f mfma(const u32x4 &a, const u32x4 &b, v16f c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
    // 16x16 tile, 32 deep: lane = 16 * (k / 8) + row (A) or column (B); result rows 4 (lane / 16) + r, column lane % 16
    __device__ static inline v4f mfma16(const u32x4 &a, const u32x4 &b, v4f c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    }
};
template <> struct Lp<bf16_t> {
    static constexpr int code = LSTM_DTYPE_BF16;
    __device__ static inline float to_f(bf16_t v) { return bf16_to_float(v); }
    // the hardware conversion (round to nearest even, NaN stays NaN): one instruction instead of five
    __device__ static inline bf16_t from_f(float v) {
        bf16_t r;
        r.bits = __builtin_bit_cast(unsigned short, (__bf16)v);
        return r;
    }
    __device__ static inline v16f mfma(const u32x4 &a, const u32x4 &b, v16f c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8b, a), __builtin_bit_cast(v8b, b), c, 0, 0, 0);
    }
    __device__ static inline v4f mfma16(const u32x4 &a, const u32x4 &b, v4f c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8b, a), __builtin_bit_cast(v8b, b), c, 0, 0, 0);
    }
};

inline size_t dtype_size(int dtype) { return dtype == LSTM_DTYPE_FP32 ? 4 : 2; }

// ---------------------------------------------------------------- device math
__device__ inline float sigmoidf_dev(float a) {
    // 1/(1+e^-a); for large |a| the exponential saturates to 0 or inf and the
    // reciprocal to 1 or 0, both correct limits.  The hardware reciprocal (1 ulp)
    // replaces the IEEE division sequence: the gate epilogues are issue-bound.
    return __builtin_amdgcn_rcpf(1.0f + __expf(-a));
}
__device__ inline float tanhf_dev(float a) {
    // tanh(a) = 1 - 2/(e^{2a}+1); exact limits at +-inf, no cancellation issue
    // beyond fp32 rounding near 0 where the result is ~a.
    float e = __expf(2.0f * a);
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}

// ---------------------------------------------------------------- optional launch timing
enum KernelClass {
    KC_GEMM_BATCHED = 0,   // whole-sequence GEMMs: input projection, dX, dW/dU
    KC_GEMM_STEP = 1,      // per-time-step recurrent GEMMs (forward and BPTT)
    KC_POINTWISE = 2,      // gate non-linearities forward / backward
    KC_AUX = 3,            // transposes, column sums, head, embedding, fills
    KC_AVERAGE = 4,        // grad_average
    KC_UPDATE = 5,         // master_update
    KC_COUNT = 6
};
bool timing_enabled();
// Brackets the launches enqueued during its lifetime with two HIP events on
// `s` when timing is enabled (lstm_timing_enable); otherwise does nothing.
class KernelTimer {
public:
    KernelTimer(int cls, hipStream_t s, double flops, double bytes);
    ~KernelTimer();
    KernelTimer(const KernelTimer &) = delete;
    KernelTimer &operator=(const KernelTimer &) = delete;
private:
    int cls_;
    hipStream_t stream_;
    void *beg_;
};

// ---------------------------------------------------------------- GEMM interface
// C[M,N] = A[M,K] * B[N,K]^T (+ bias[N]) ; both operands K-contiguous.
struct GemmArgs {
    const void *A;      // lp [M, lda]
    const void *B;      // lp [N, ldb]
    void *C;            // fp32 or lp [M, ldc]
    const void *bias;   // lp [N] or null
    int M, N, K;
    int64_t lda, ldb, ldc;
    int out_lp;         // 1: C is lp, 0: C is fp32
    int accumulate;     // fp32 C only: C += result
    float *splitk_ws;   // non-null with splits > 1: fp32 [splits, M, N] partials
    int splits;
    int kclass;         // KernelClass the launch is accounted to
};

// Enqueue one GEMM. dtype = LSTM_DTYPE_*. Returns LSTM_OK or an error status.
int gemm_nt(int dtype, const GemmArgs &g, hipStream_t stream);
// C[M,N] = A^T B with A[K,M] (lda) and B[K,N] (ldb): contraction over the rows of both
// operands, no transposed copies.  16-bit types, aligned shapes with M, N >= 192 only.
bool gemm_tn_supported(int dtype, const GemmArgs &g);
int gemm_tn(int dtype, const GemmArgs &g, hipStream_t stream);
// ---- operands in 64x64 blocks: tensor [R, C] stored as [ceil(R/64)][ncb][64][64], zero padded.
// A view may start at any row block (ptr points at that block row).
struct BlockedOperand {
    const void *ptr;
    int ncb;      // column blocks per row block (>= ceil(C/64))
    int trans;    // 0: rows index M (resp. N), columns index K; 1: rows index K, columns index M (resp. N)
    int packed = 0;   // 1: every 64x64 block in MFMA-fragment order (packed.h, two 32-row blocks) instead of row-major:
                      //    the per-time-step copies the recurrent kernels write, one after the other.  gemm_stream_tn only
};
struct BlockedGemmArgs {
    BlockedOperand A, B;
    void *C;             // row-major fp32 or lp [M, ldc]
    const void *bias;    // lp [N] or null
    int M, N, K;
    int64_t ldc;
    int out_lp, accumulate;
    float *splitk_ws;
    int splits;
    int kclass;
    // batch > 1 (both operands in the rows-are-K role): `batch` products whose K rows interleave in
    // memory in segments of seg_len block rows: K tile t of product y is block row
    // (t / seg_len) * seg_stride + t % seg_len + y * seg_len; results batch_c elements apart.
    int batch = 1, seg_len = 0, seg_stride = 0;
    int64_t batch_c = 0;
    // batch > 1 only: a second product with the same A in the same launch, C2 [M, ldc2] = A^T B2 with N2 columns (same
    // roles, batch layout and batch_c as B / C).  dW and dU of a layer share dA: issued together, the tiles of both
    // run side by side on one XCD and dA comes from memory once.  B2.ptr null: none.
    BlockedOperand B2{nullptr, 0, 1, 0};
    void *C2 = nullptr;
    int64_t ldc2 = 0;
    int N2 = 0;
};
size_t blocked_elems(int rows, int cols);
// dst (blocked, zero padded) = src (row-major [rows, cols], leading dimension ld)
int pack_blocked(int dtype, const void *src, int64_t ld, int rows, int cols, void *dst, hipStream_t stream);
bool gemm_blocked_supported(int dtype, int M, int N);
// 16-bit C [M, ldc] = sum of `splits` fp32 partial results ws [split][M][N], added up in index order
int splitk_reduce(int dtype, const float *ws, int splits, int M, int N, void *C, int64_t ldc, hipStream_t stream);
// C = op(A) op(B)^T-style product of blocked operands (roles per BlockedOperand::trans);
// supported role pairs: (0,0), (0,1), (1,1).
int gemm_blocked(int dtype, const BlockedGemmArgs &g, hipStream_t stream);
// ---- operands in packed (MFMA-fragment) order (packed.h): C[M,N] (+ bias) = A B^T, 16-bit row-major result.
// A: the rows of `rows_per_step` consecutive rows form one time step, stored as [64-row tile][K/64][A chunk],
//    consecutive time steps a_step_stride elements apart.  B: [128-row tile][K/64][B chunk].
struct StreamGemmArgs {
    const void *A;
    int64_t a_step_stride;
    int rows_per_step;
    const void *B;
    void *C;
    int64_t ldc;
    const void *bias;    // [N] or null
    int M, N, K;
    int gate_h;          // 0: row n of B is column n of C.  H: row 32 g + r of B tile j is column g H + 32 j + r (N = 4H)
    int kclass;
};
bool gemm_stream_supported(int dtype, const StreamGemmArgs &g);
int gemm_stream(int dtype, const StreamGemmArgs &g, hipStream_t stream);
// The (1,1) role pair of gemm_blocked (C = A^T B, 16-bit result, no bias, one product, no split) on the kernel of
// gemm_stream.hip; K a multiple of 128.
bool gemm_stream_tn_supported(int dtype, const BlockedGemmArgs &g);
int gemm_stream_tn(int dtype, const BlockedGemmArgs &g, hipStream_t stream);
// number of K splits gemm_nt / gemm_tn would like for this shape (>= 1)
// Diagnostic MFMA loop: operands = 256*512*2 16-byte fragments (device), sink = 1 float (device).
int mfma_rate(int dtype, const void *operands, int iters, float *sink, double *flops, hipStream_t stream);
int gemm_pick_splits(int dtype, int M, int N, int K);

}  // namespace lstm
