// GEMM kernels: C[M,N] = A[M,K] * B[N,K]^T, both operands K-contiguous.
//
//  * half / bfloat16: LDS-staged tiles feeding v_mfma_f32_32x32x16 (fp32
//    accumulate), 4 wavefronts of 64 lanes per workgroup, each owning a 64x64
//    sub-tile as 2x2 MFMA blocks.
//  * fp32 (the all-single-precision baseline mode): LDS-tiled FMA kernel.
//
// Optional bias add, fp32 accumulate-into-C, low-precision output, and a
// split-K form writing fp32 partials that a second kernel sums in a fixed
// order (deterministic).
#include "common.h"

namespace lstm {

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_PAD = 8;               // 16 bytes per row: spreads 16-byte reads over the banks
constexpr int LDS_LD = BK + LDS_PAD;     // elements per LDS row
constexpr int THREADS = 256;

struct KernArgs {
    const void *A;
    const void *B;
    void *C;
    const void *bias;
    int M, N, K;
    int64_t lda, ldb, ldc;
    int out_lp, accumulate;
    float *ws;          // split-K partials or null
    int k_chunk;        // K range handled by one blockIdx.z
    int vec_ok;         // rows 16-byte aligned and K % 8 == 0: 16-byte global loads allowed
};

// 16-byte global load of 8 lp elements of row `row` at column k; zero outside.
template <typename T>
__device__ inline uint4 load8(const T *base, int64_t ld, int row, int nrows, int k, int kend, int vec_ok) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row >= nrows || k >= kend) return v;
    const T *p = base + (int64_t)row * ld + k;
    if (vec_ok && k + 8 <= kend) {
        v = *reinterpret_cast<const uint4 *>(p);
    } else {
        uint16_t tmp[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) tmp[j] = (k + j < kend) ? reinterpret_cast<const uint16_t *>(p)[j] : (uint16_t)0;
        v.x = tmp[0] | ((uint32_t)tmp[1] << 16);
        v.y = tmp[2] | ((uint32_t)tmp[3] << 16);
        v.z = tmp[4] | ((uint32_t)tmp[5] << 16);
        v.w = tmp[6] | ((uint32_t)tmp[7] << 16);
    }
    return v;
}

template <typename T>
__global__ __launch_bounds__(THREADS) void gemm_nt_mfma_kernel(KernArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDS_LD];

    const T *A = reinterpret_cast<const T *>(a.A);
    const T *B = reinterpret_cast<const T *>(a.B);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // each thread moves 4 + 4 vectors of 8 elements per K tile
    uint4 ra[4], rb[4];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int v = tid + THREADS * i;
            int row = v >> 3, kv = (v & 7) * 8;
            ra[i] = load8<T>(A, a.lda, m0 + row, a.M, k0 + kv, kend, a.vec_ok);
            rb[i] = load8<T>(B, a.ldb, n0 + row, a.N, k0 + kv, kend, a.vec_ok);
        }
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int v = tid + THREADS * i;
            int row = v >> 3, kv = (v & 7) * 8;
            *reinterpret_cast<uint4 *>(&As[buf][row * LDS_LD + kv]) = ra[i];
            *reinterpret_cast<uint4 *>(&Bs[buf][row * LDS_LD + kv]) = rb[i];
        }
    };

    const int ntiles = (kend > kbeg) ? (kend - kbeg + BK - 1) / BK : 0;
    if (ntiles > 0) {
        gload(kbeg);
        sstore(0);
    }
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) gload(kbeg + (t + 1) * BK);
        const int lrow = lane & 31, lk = (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            uint4 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = *reinterpret_cast<const uint4 *>(&As[buf][(wm * 64 + i * 32 + lrow) * LDS_LD + ks * 16 + lk]);
                fb[i] = *reinterpret_cast<const uint4 *>(&Bs[buf][(wn * 64 + i * 32 + lrow) * LDS_LD + ks * 16 + lk]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = Lp<T>::mfma(fa[i], fb[j], acc[i][j]);
        }
        if (t + 1 < ntiles) sstore(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds, for each 32x32 block, column (lane%32) and rows
    // 8*(r/4) + 4*(lane/32) + r%4, r = 0..15
    const int col_l = lane & 31, rgrp = (lane >> 5) * 4;
    const T *bias = reinterpret_cast<const T *>(a.bias);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + col_l;
            if (col >= a.N) continue;
            const float bv = (bias && blockIdx.z == 0) ? Lp<T>::to_f(bias[col]) : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 64 + i * 32 + (r >> 2) * 8 + rgrp + (r & 3);
                if (row >= a.M) continue;
                float v = acc[i][j][r] + bv;
                if (a.ws) {
                    a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
                } else if (a.out_lp) {
                    reinterpret_cast<T *>(a.C)[(int64_t)row * a.ldc + col] = Lp<T>::from_f(v);
                } else {
                    float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
                    *c = a.accumulate ? (*c + v) : v;
                }
            }
        }
}

// fp32 baseline-mode GEMM: 64x64 tile, 16-deep K slices, 4x4 outputs per thread.
constexpr int SBM = 64, SBN = 64, SBK = 16;
__global__ __launch_bounds__(256) void gemm_nt_f32_kernel(KernArgs a) {
    __shared__ float As[SBK][SBM + 1];
    __shared__ float Bs[SBK][SBN + 1];
    const float *A = reinterpret_cast<const float *>(a.A);
    const float *B = reinterpret_cast<const float *>(a.B);
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * SBM, n0 = blockIdx.x * SBN;
    const int kbeg = blockIdx.z * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);
    float acc[4][4] = {};
    for (int k0 = kbeg; k0 < kend; k0 += SBK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = tid + 256 * i;          // 0..1023 over a 64 x 16 slice
            int row = e >> 4, kk = e & 15;
            int k = k0 + kk;
            As[kk][row] = (m0 + row < a.M && k < kend) ? A[(int64_t)(m0 + row) * a.lda + k] : 0.0f;
            Bs[kk][row] = (n0 + row < a.N && k < kend) ? B[(int64_t)(n0 + row) * a.ldb + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < SBK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
    const float *bias = reinterpret_cast<const float *>(a.bias);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = m0 + ty * 4 + i;
        if (row >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = n0 + tx * 4 + j;
            if (col >= a.N) continue;
            float v = acc[i][j] + ((bias && blockIdx.z == 0) ? bias[col] : 0.0f);
            if (a.ws) {
                a.ws[((int64_t)blockIdx.z * a.M + row) * a.N + col] = v;
            } else {
                float *c = reinterpret_cast<float *>(a.C) + (int64_t)row * a.ldc + col;
                *c = a.accumulate ? (*c + v) : v;
            }
        }
    }
}

// sum split-K partials in index order and store
template <typename T>
__global__ void splitk_reduce_kernel(const float *ws, int splits, int M, int N, void *C, int64_t ldc, int out_lp,
                                     int accumulate) {
    const int64_t total = (int64_t)M * N;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int z = 0; z < splits; ++z) s += ws[(int64_t)z * total + e];
        const int row = (int)(e / N), col = (int)(e % N);
        if (out_lp) {
            reinterpret_cast<T *>(C)[(int64_t)row * ldc + col] = Lp<T>::from_f(s);
        } else {
            float *c = reinterpret_cast<float *>(C) + (int64_t)row * ldc + col;
            *c = accumulate ? (*c + s) : s;
        }
    }
}

template <typename T>
int launch(const GemmArgs &g, hipStream_t stream) {
    constexpr bool is_f32 = sizeof(T) == 4;
    const int bm = is_f32 ? SBM : BM, bn = is_f32 ? SBN : BN, bk = is_f32 ? SBK : BK;
    KernArgs a;
    a.A = g.A; a.B = g.B; a.C = g.C; a.bias = g.bias;
    a.M = g.M; a.N = g.N; a.K = g.K;
    a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
    a.out_lp = g.out_lp; a.accumulate = g.accumulate;
    int splits = (g.splitk_ws && g.splits > 1) ? g.splits : 1;
    int k_chunk = g.K;
    if (splits > 1) {
        k_chunk = ((g.K + splits - 1) / splits + bk - 1) / bk * bk;
        splits = (g.K + k_chunk - 1) / k_chunk;
    }
    a.ws = splits > 1 ? g.splitk_ws : nullptr;
    a.k_chunk = k_chunk;
    a.vec_ok = (!is_f32 && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
                ((uintptr_t)g.A % 16 == 0) && ((uintptr_t)g.B % 16 == 0)) ? 1 : 0;
    dim3 grid((g.N + bn - 1) / bn, (g.M + bm - 1) / bm, splits);
    if (grid.y > 65535u || grid.z > 65535u) {
        set_error("gemm_nt: grid too large (M=%d splits=%d)", g.M, splits);
        return LSTM_ERR_UNSUPPORTED;
    }
    KernelTimer timer(g.kclass, stream, 2.0 * g.M * g.N * g.K, 0.0);
    if constexpr (is_f32) {
        hipLaunchKernelGGL(gemm_nt_f32_kernel, grid, dim3(256), 0, stream, a);
    } else {
        hipLaunchKernelGGL(gemm_nt_mfma_kernel<T>, grid, dim3(THREADS), 0, stream, a);
    }
    LSTM_LAUNCH_CHECK();
    if (splits > 1) {
        const int64_t total = (int64_t)g.M * g.N;
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(splitk_reduce_kernel<T>, dim3(blocks), dim3(256), 0, stream, g.splitk_ws, splits, g.M, g.N,
                           g.C, g.ldc, g.out_lp, g.accumulate);
        LSTM_LAUNCH_CHECK();
    }
    return LSTM_OK;
}

}  // namespace

int gemm_pick_splits(int M, int N, int K) {
    // enough workgroups to cover the 256 compute units a few times over
    const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    if (tiles >= 512 || K < 4 * BK) return 1;
    long want = (1024 + tiles - 1) / tiles;
    long maxs = K / (2 * BK);
    if (want > maxs) want = maxs;
    if (want > 256) want = 256;
    return want < 1 ? 1 : (int)want;
}

int gemm_nt(int dtype, const GemmArgs &g, hipStream_t stream) {
    if (g.M <= 0 || g.N <= 0) return LSTM_OK;
    if (!g.A || !g.B || !g.C || g.K < 0) {
        set_error("gemm_nt: null operand");
        return LSTM_ERR_INVALID;
    }
    switch (dtype) {
        case LSTM_DTYPE_FP32: return launch<float>(g, stream);
        case LSTM_DTYPE_FP16: return launch<_Float16>(g, stream);
        case LSTM_DTYPE_BF16: return launch<bf16_t>(g, stream);
    }
    set_error("gemm_nt: bad dtype %d", dtype);
    return LSTM_ERR_INVALID;
}

}  // namespace lstm
