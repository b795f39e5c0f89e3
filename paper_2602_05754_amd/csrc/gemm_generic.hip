// Edge-safe grouped GEMM on plain fp32 FMAs (no matrix cores).
//
// Serves the fp32 configuration (true fp32 arithmetic, needed for the 1e-5
// parity bound) and any bf16 problem whose dimensions the MFMA kernel does not
// take.  Computes both halves of a backward action (TimelyFreeze Sec. 3.2.1):
// the input gradient dX = dY W^T (layout kNT) and the parameter gradient
// dW = X^T dY (layout kTN); frozen tensors never reach this file.
//
// 64 x 64 output tile per 256-thread block, 4 x 4 outputs per thread,
// contraction staged through LDS 16 at a time.
#include "tf_internal.h"

namespace tf {
namespace {

constexpr int kTile = 64;
constexpr int kBK = 16;
constexpr int kThreads = 256;

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t x) {
    return __uint_as_float(uint32_t(x) << 16);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// kContig: the contraction index is the fast (contiguous) index of A and B.
template <typename TIn, bool kContig, bool kOutBf16, bool kAccumulate>
__global__ __launch_bounds__(kThreads) void gemm_generic_kernel(GemmBatch batch) {
    __shared__ float As[kBK][kTile + 4];
    __shared__ float Bs[kBK][kTile + 4];

    int pi = 0;
    const int bid = blockIdx.x;
    for (int i = 1; i < batch.n_problems; ++i)
        if (bid >= batch.p[i].tile_start) pi = i;
    const GemmProblem& P = batch.p[pi];
    const int M = P.M, N = P.N, Kc = P.Kc;
    const int tiles_n = (N + kTile - 1) / kTile;
    const int t = bid - P.tile_start;
    const int m0 = (t / tiles_n) * kTile;
    const int n0 = (t % tiles_n) * kTile;
    const TIn* A = static_cast<const TIn*>(P.A);
    const TIn* B = static_cast<const TIn*>(P.B);

    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;      // 16 x 16 threads, 4 x 4 outputs each
    float acc[4][4] = {};

    for (int k0 = 0; k0 < Kc; k0 += kBK) {
        // stage A(m0.., k0..) and B(n0.., k0..) into LDS as [k][row]
#pragma unroll
        for (int i = 0; i < (kTile * kBK) / kThreads; ++i) {
            const int idx = tid + i * kThreads;
            int r, k;
            if (kContig) { k = idx % kBK; r = idx / kBK; }    // consecutive threads walk the contraction
            else         { r = idx % kTile; k = idx / kTile; }  // consecutive threads walk the rows
            const int gk = k0 + k;
            float a = 0.f, b = 0.f;
            if (gk < Kc) {
                if (m0 + r < M)
                    a = to_f32<TIn>(kContig ? A[int64_t(m0 + r) * P.lda + gk] : A[int64_t(gk) * P.lda + (m0 + r)]);
                if (n0 + r < N)
                    b = to_f32<TIn>(kContig ? B[int64_t(n0 + r) * P.ldb + gk] : B[int64_t(gk) * P.ldb + (n0 + r)]);
            }
            As[k][r] = a;
            Bs[k][r] = b;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kBK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            const int64_t off = int64_t(m) * N + n;
            if (kOutBf16) {
                static_cast<uint16_t*>(P.C)[off] = f32_to_bf16_rne(acc[i][j]);
            } else {
                float* c = static_cast<float*>(P.C) + off;
                *c = kAccumulate ? (*c + acc[i][j]) : acc[i][j];
            }
        }
    }
}

template <typename TIn, bool kContig>
void dispatch_out(hipStream_t stream, const GemmBatch& batch, Dtype out_dtype, bool accumulate) {
    const dim3 grid(batch.total_tiles), block(kThreads);
    if (out_dtype == Dtype::BF16)
        hipLaunchKernelGGL((gemm_generic_kernel<TIn, kContig, true, false>), grid, block, 0, stream, batch);
    else if (accumulate)
        hipLaunchKernelGGL((gemm_generic_kernel<TIn, kContig, false, true>), grid, block, 0, stream, batch);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<TIn, kContig, false, false>), grid, block, 0, stream, batch);
}

}  // namespace

int gemm_generic_tile() { return kTile; }

hipError_t launch_gemm_generic(hipStream_t stream, GemmBatch& batch, int n_problems,
                               Layout layout, Dtype in_dtype, Dtype out_dtype, bool accumulate) {
    batch.n_problems = n_problems;
    if (n_problems == 0 || batch.total_tiles == 0) return hipSuccess;
    const bool contig = layout == Layout::kNT;
    if (in_dtype == Dtype::F32) {
        if (contig) dispatch_out<float, true>(stream, batch, out_dtype, accumulate);
        else        dispatch_out<float, false>(stream, batch, out_dtype, accumulate);
    } else {
        if (contig) dispatch_out<uint16_t, true>(stream, batch, out_dtype, accumulate);
        else        dispatch_out<uint16_t, false>(stream, batch, out_dtype, accumulate);
    }
    return hipGetLastError();
}

}  // namespace tf
