// Grouped bf16 GEMM on the gfx950 matrix cores for the two halves of a backward
// action (TimelyFreeze Sec. 3.2.1):
//   kNT  dX = dY W^T   - contraction (N_l) is the contiguous index of both inputs
//   kTN  dW = X^T dY   - contraction (T) is the slow index of both inputs
// Only tensors that are not frozen are ever listed in a kTN batch, so a frozen
// tensor's dW tiles cost nothing and its buffers are never touched.
//
// One 256 x 256 output tile per 256-thread workgroup (4 wave64s in a 2 x 2
// grid, 128 x 128 per wave = 4 x 4 MFMA 32x32x16 tiles, 256 fp32 accumulators
// per lane).  The contraction advances 64 at a time through two LDS stages of
// 64 KB.  Both layouts put their operands into LDS in the same form,
// [row][64 contraction values] with the eight 16-byte chunks of a row XOR-
// swizzled, so the MFMA loop is shared; kTN transposes 8 x 8 blocks in
// registers on the way in.
#include "tf_internal.h"

namespace tf {
namespace {

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kThreads = 256;
constexpr int kRowBytes = kBK * 2;                    // 128 B of contraction per tile row
constexpr int kTileBytes = kBM * kRowBytes;           // 32 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;           // A + B
constexpr int kLdsBytes = 2 * kStageBytes;            // two stages = 128 KB
constexpr int kGroupM = 8;                            // tile rows per L2 locality group
constexpr int kXcds = 8;
constexpr int kXcdRun = 32;                           // consecutive logical tiles kept on one XCD

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
struct alignas(16) U4 { uint32_t x, y, z, w; };
struct alignas(8) U2 { uint32_t x, y; };
struct alignas(16) F4 { float x, y, z, w; };

// 16-byte chunk c (0..7) of tile row `row` lives at chunk c ^ swz(row).  Rows r..r+7
// (MFMA reads) and rows 8q+j for q..q+7 (transposing writes) both spread over all 8 chunks.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a = ((a & 0x7fffffffu) > 0x7f800000u) ? ((a >> 16) | 0x40u) : ((a + 0x7fffu + ((a >> 16) & 1u)) >> 16);
    b = ((b & 0x7fffffffu) > 0x7f800000u) ? ((b >> 16) | 0x40u) : ((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
    return (a & 0xffffu) | (b << 16);
}

// ---- global -> registers -------------------------------------------------------------------
// kNT: src is [rows x Kc]; thread reads chunk (tid % 8) of rows tid/8 + 32 p.
__device__ __forceinline__ void gload_nt(const uint16_t* src, int64_t ld, int row0, int k0, U4 (&r)[8]) {
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
    const uint16_t* base = src + int64_t(row0 + rr) * ld + k0 + c * 8;
#pragma unroll
    for (int p = 0; p < 8; ++p) r[p] = *reinterpret_cast<const U4*>(base + int64_t(32 * p) * ld);
}
__device__ __forceinline__ void lstore_nt(char* tile, const U4 (&r)[8]) {
    const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int row = rr + 32 * p;
        *reinterpret_cast<U4*>(tile + row * kRowBytes + ((c ^ swz(row)) << 4)) = r[p];
    }
}

// kTN: src is [Kc x rows]; thread reads 8 consecutive rows-of-the-tile (one 16-byte chunk)
// at contraction indices k0 + 8 tg + j, j = 0..7, with tg = tid / 32, chunk mc = tid % 32.
__device__ __forceinline__ void gload_tn(const uint16_t* src, int64_t ld, int row0, int k0, U4 (&r)[8]) {
    const int mc = threadIdx.x & 31, tg = threadIdx.x >> 5;
    const uint16_t* base = src + int64_t(k0 + tg * 8) * ld + row0 + mc * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = *reinterpret_cast<const U4*>(base + int64_t(j) * ld);
}
__device__ __forceinline__ void lstore_tn(char* tile, const U4 (&r)[8]) {
    const int mc = threadIdx.x & 31, tg = threadIdx.x >> 5;
    // 8 x 8 transpose of 16-bit values: r[j] holds 8 tile rows at contraction j;
    // o[i] holds 8 contraction values of tile row i.
    const uint32_t* in = reinterpret_cast<const uint32_t*>(&r[0]);   // in[j*4 + d]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t a = in[(2 * q) * 4 + (i >> 1)], b = in[(2 * q + 1) * 4 + (i >> 1)];
            o[q] = (i & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
        }
        const int row = mc * 8 + i;
        *reinterpret_cast<U4*>(tile + row * kRowBytes + ((tg ^ swz(row)) << 4)) = U4{o[0], o[1], o[2], o[3]};
    }
}

template <bool kTN>
__device__ __forceinline__ void gload(const uint16_t* A, const uint16_t* B, int64_t lda, int64_t ldb,
                                      int m0, int n0, int k0, U4 (&ra)[8], U4 (&rb)[8]) {
    if (kTN) { gload_tn(A, lda, m0, k0, ra); gload_tn(B, ldb, n0, k0, rb); }
    else     { gload_nt(A, lda, m0, k0, ra); gload_nt(B, ldb, n0, k0, rb); }
}
template <bool kTN>
__device__ __forceinline__ void lstore(char* stage, const U4 (&ra)[8], const U4 (&rb)[8]) {
    if (kTN) { lstore_tn(stage, ra); lstore_tn(stage + kTileBytes, rb); }
    else     { lstore_nt(stage, ra); lstore_nt(stage + kTileBytes, rb); }
}

// blockIdx -> logical tile.  Hardware hands workgroup b to XCD b % 8; runs of kXcdRun
// consecutive logical tiles are kept on one XCD (shared L2), runs go round-robin over
// the XCDs so that all of them work on the same part of the tile list.
__device__ __forceinline__ int logical_tile(int b, int nb) {
    const int span = kXcds * kXcdRun;
    const int full = (nb / span) * span;
    if (b >= full) return b;
    const int xcd = b % kXcds, idx = b / kXcds;
    return ((idx / kXcdRun) * kXcds + xcd) * kXcdRun + idx % kXcdRun;
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
__global__ __launch_bounds__(kThreads) void gemm_mfma_kernel(GemmBatch batch) {
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int lt = logical_tile(blockIdx.x, gridDim.x);
    int pi = 0;
    for (int i = 1; i < batch.n_problems; ++i)
        if (lt >= batch.p[i].tile_start) pi = i;
    const GemmProblem& P = batch.p[pi];
    const int M = P.M, N = P.N, Kc = P.Kc;
    const int tiles_m = M / kBM, tiles_n = N / kBN;
    int t = lt - P.tile_start;
    const int per_group = kGroupM * tiles_n;
    const int first_m = (t / per_group) * kGroupM;
    const int gsz = min(tiles_m - first_m, kGroupM);
    t %= per_group;
    const int m0 = (first_m + t % gsz) * kBM;
    const int n0 = (t / gsz) * kBN;

    const uint16_t* A = static_cast<const uint16_t*>(P.A);
    const uint16_t* B = static_cast<const uint16_t*>(P.B);
    const int64_t lda = kTN ? M : Kc, ldb = kTN ? N : Kc;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    U4 ra[8], rb[8];
    const int nk = Kc / kBK;
    gload<kTN>(A, B, lda, ldb, m0, n0, 0, ra, rb);
    lstore<kTN>(lds, ra, rb);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        char* cur = lds + (kt & 1) * kStageBytes;
        char* nxt = lds + ((kt + 1) & 1) * kStageBytes;
        const bool more = kt + 1 < nk;
        if (more) gload<kTN>(A, B, lda, ldb, m0, n0, (kt + 1) * kBK, ra, rb);

        const char* tA = cur + (wm * 128 + lrow) * kRowBytes;
        const char* tB = cur + kTileBytes + (wn * 128 + lrow) * kRowBytes;
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
            bf16x8 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rowa = wm * 128 + i * 32 + lrow, rowb = wn * 128 + i * 32 + lrow;
                fa[i] = *reinterpret_cast<const bf16x8*>(tA + i * 32 * kRowBytes + (((2 * s + lhalf) ^ swz(rowa)) << 4));
                fb[i] = *reinterpret_cast<const bf16x8*>(tB + i * 32 * kRowBytes + (((2 * s + lhalf) ^ swz(rowb)) << 4));
            }
            // D rows <- n (B operand rows), D columns <- m: a lane then owns 4 consecutive n
            // of one output row m, i.e. 4 contiguous elements of row-major C.
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }

        if (more) lstore<kTN>(nxt, ra, rb);
        __syncthreads();
    }

    // epilogue: acc[i][j][4g + e] is C[m][n] with m = m0 + wm*128 + i*32 + lane%32,
    // n = n0 + wn*128 + j*32 + 8g + 4*(lane/32) + e.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + wm * 128 + i * 32 + lrow;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * 128 + j * 32 + 8 * g + 4 * lhalf;
                const int64_t off = m * N + n;
                const float c0 = acc[i][j][4 * g + 0], c1 = acc[i][j][4 * g + 1];
                const float c2 = acc[i][j][4 * g + 2], c3 = acc[i][j][4 * g + 3];
                if (kOutBf16) {
                    *reinterpret_cast<U2*>(static_cast<uint16_t*>(P.C) + off) =
                        U2{f32x2_to_bf16x2(c0, c1), f32x2_to_bf16x2(c2, c3)};
                } else {
                    F4* dst = reinterpret_cast<F4*>(static_cast<float*>(P.C) + off);
                    if (kAccumulate) {
                        const F4 old = *dst;
                        *dst = F4{old.x + c0, old.y + c1, old.z + c2, old.w + c3};
                    } else {
                        *dst = F4{c0, c1, c2, c3};
                    }
                }
            }
        }
    }
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
hipError_t launch_one(hipStream_t stream, const GemmBatch& batch) {
    auto kern = gemm_mfma_kernel<kTN, kOutBf16, kAccumulate>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(batch.total_tiles), dim3(kThreads), kLdsBytes, stream, batch);
    return hipGetLastError();
}

}  // namespace

int gemm_mfma_tile() { return kBM; }

bool mfma_shape_ok(int64_t M, int64_t N, int64_t Kc) {
    return M > 0 && N > 0 && Kc > 0 && M % kBM == 0 && N % kBN == 0 && Kc % kBK == 0;
}

hipError_t launch_gemm_mfma_bf16(hipStream_t stream, GemmBatch& batch, int n_problems,
                                 Layout layout, Dtype out_dtype, bool accumulate) {
    batch.n_problems = n_problems;
    if (n_problems == 0 || batch.total_tiles == 0) return hipSuccess;
    const bool tn = layout == Layout::kTN;
    if (out_dtype == Dtype::BF16)
        return tn ? launch_one<true, true, false>(stream, batch) : launch_one<false, true, false>(stream, batch);
    if (accumulate)
        return tn ? launch_one<true, false, true>(stream, batch) : launch_one<false, false, true>(stream, batch);
    return tn ? launch_one<true, false, false>(stream, batch) : launch_one<false, false, false>(stream, batch);
}

}  // namespace tf
