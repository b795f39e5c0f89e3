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
// 64 KB that are filled by direct global->LDS loads (no register staging):
// while the matrix cores work on one stage the next one is in flight.
//
//   kNT stage: [256 rows][64 contraction] per operand, 16-byte chunks of a row
//              XOR-swizzled; MFMA operands are plain 128-bit LDS reads.
//   kTN stage: [64 contraction][256 rows] per operand (the layout in memory),
//              64-byte blocks of a row XOR-swizzled; MFMA operands come from the
//              LDS transpose read (4 contraction values of one row per lane).
// A direct-to-LDS load writes lane i's 16 bytes at (wave-uniform base) + 16 i,
// so a swizzle is applied by choosing which global address each lane fetches.
#include "tf_internal.h"

namespace tf {
namespace {

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kThreads = 256;
constexpr int kTileBytes = kBM * kBK * 2;             // 32 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;           // A + B
constexpr int kLdsBytes = 2 * kStageBytes;            // two stages = 128 KB
constexpr int kGroupM = 8;                            // tile rows per L2 locality group
constexpr int kXcds = 8;
constexpr int kXcdRun = 32;                           // consecutive logical tiles kept on one XCD

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));
typedef float F4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4* LdsBf16x4Ptr;

#define TF_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define TF_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a = ((a & 0x7fffffffu) > 0x7f800000u) ? ((a >> 16) | 0x40u) : ((a + 0x7fffu + ((a >> 16) & 1u)) >> 16);
    b = ((b & 0x7fffffffu) > 0x7f800000u) ? ((b >> 16) | 0x40u) : ((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
    return (a & 0xffffu) | (b << 16);
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

// ---------------------------------------------------------------------------------------------
// Stage fill.  Each wave issues 8 direct-to-LDS loads per operand; load p of wave w fills the
// 1 KB of the operand tile at (4 p + w) KB.
//   kNT: that KB is tile rows R = 32 p + 8 w + lane/8, physical chunk lane%8 of each row;
//        logical chunk = physical ^ ((R ^ (R >> 3)) & 7).
//   kTN: that KB is contraction rows T = 8 p + 2 w + lane/32, 16-byte slot lane%32 of each;
//        logical 64-byte block = physical block ^ (T & 3).
// ---------------------------------------------------------------------------------------------
struct FillPtrs {
    const char* a[2];         // per-lane global byte pointers of load p = 0 (and p = 1 for kNT)
    const char* b[2];
    int64_t step_a, step_b;   // byte distance between loads p and p + 2 (kNT) / p and p + 1 (kTN)
};

template <bool kTN>
__device__ __forceinline__ FillPtrs make_fill(const uint16_t* A, const uint16_t* B, int64_t lda, int64_t ldb,
                                              int m0, int n0) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    FillPtrs f;
    if (kTN) {
        const int T = 2 * w + (lane >> 5);                     // + 8 p
        const int slot = lane & 31;
        const int blk = (slot >> 2) ^ (T & 3);
        const int col = blk * 32 + (slot & 3) * 8;             // element offset inside the 256-wide tile row
        f.a[0] = reinterpret_cast<const char*>(A + int64_t(T) * lda + m0 + col);
        f.b[0] = reinterpret_cast<const char*>(B + int64_t(T) * ldb + n0 + col);
        f.a[1] = f.a[0]; f.b[1] = f.b[0];
        f.step_a = 8 * lda * 2; f.step_b = 8 * ldb * 2;
    } else {
        const int r = 8 * w + (lane >> 3);                     // + 32 p
        const int pc = lane & 7;
#pragma unroll
        for (int q = 0; q < 2; ++q) {                          // p even / odd differ in bit 2 of the swizzle
            const int R = r + 32 * q;
            const int c = pc ^ ((R ^ (R >> 3)) & 7);
            f.a[q] = reinterpret_cast<const char*>(A + int64_t(m0 + R) * lda + c * 8);
            f.b[q] = reinterpret_cast<const char*>(B + int64_t(n0 + R) * ldb + c * 8);
        }
        f.step_a = 64 * lda * 2; f.step_b = 64 * ldb * 2;
    }
    return f;
}

// One direct-to-LDS load: every lane fetches 16 bytes from its own global address and the
// wave's 1 KB lands at LDS byte address lds_base (wave-uniform, goes through M0) + 16 * lane.
// Written as inline assembly so that the compiler's wait-count insertion does not treat every
// later LDS read as dependent on it (it would drain the load queue before each transpose read);
// completion is awaited explicitly with wait_direct_loads() before the stage barrier.
__device__ __forceinline__ void direct_load_16B(const char* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base), "v"(gptr)
                 : "memory");
}
__device__ __forceinline__ void wait_direct_loads() {
    __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0), other counters untouched
}

// Issue load number q (0..15) of a stage fill: even q fetch operand A, odd q operand B, load p = q / 2.
template <bool kTN>
__device__ __forceinline__ void fill_one(const FillPtrs& f, int64_t koff_a, int64_t koff_b, uint32_t stage_lds, int q) {
    const uint32_t w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = q >> 1;
    if ((q & 1) == 0) {
        const char* ga = kTN ? f.a[0] + koff_a + p * f.step_a : f.a[p & 1] + koff_a + (p >> 1) * f.step_a;
        direct_load_16B(ga, stage_lds + w * 1024 + p * 4096);
    } else {
        const char* gb = kTN ? f.b[0] + koff_b + p * f.step_b : f.b[p & 1] + koff_b + (p >> 1) * f.step_b;
        direct_load_16B(gb, stage_lds + kTileBytes + w * 1024 + p * 4096);
    }
}

template <bool kTN>
__device__ __forceinline__ void fill_stage(const FillPtrs& f, int64_t koff_a, int64_t koff_b, uint32_t stage) {
#pragma unroll
    for (int q = 0; q < 16; ++q) fill_one<kTN>(f, koff_a, koff_b, stage, q);
}

// ---------------------------------------------------------------------------------------------
// MFMA operand fetch for contraction step s (16 values) of the current stage.
// Operand lane l holds row (l % 32) of a 32-row block and contraction values 8 (l / 32) .. + 7.
// ---------------------------------------------------------------------------------------------
struct FragAddr {
    int a[4], b[4];       // per-lane LDS byte offsets (inside a stage) of the 4 row blocks, step 0
};

template <bool kTN>
__device__ __forceinline__ FragAddr make_frag_addr(int wm, int wn) {
    const int lane = threadIdx.x & 63;
    FragAddr fa;
    if (kTN) {
        // 16-lane group G reads rows 8 (G / 2) + {0..3} (+4 for the second read) of the
        // contraction and columns 16 (G % 2) + {0..15} of the 32-row block; as a source lane
        // ii of its group it fetches row ii / 4, columns 4 (ii % 4) .. + 3.
        const int G = lane >> 4, ii = lane & 15;
        const int x = ii >> 2;
        const int laneoff = (8 * (G >> 1) + x) * 512 + 32 * (G & 1) + 8 * (ii & 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa.a[i] = laneoff + wm * 256 + ((i ^ x) * 64);
            fa.b[i] = kTileBytes + laneoff + wn * 256 + ((i ^ x) * 64);
        }
    } else {
        const int lrow = lane & 31, lhalf = lane >> 5;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ra = wm * 128 + i * 32 + lrow, rb = wn * 128 + i * 32 + lrow;
            // chunk (2 s + lhalf) ^ swz(row): the s-dependent part is XORed in at use
            fa.a[i] = ra * 128 + ((lhalf ^ ((ra ^ (ra >> 3)) & 7)) << 4);
            fa.b[i] = kTileBytes + rb * 128 + ((lhalf ^ ((rb ^ (rb >> 3)) & 7)) << 4);
        }
    }
    return fa;
}

template <bool kTN>
__device__ __forceinline__ bf16x8 load_frag(const char* stage, int addr, int s) {
    if (kTN) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (LdsBf16x4Ptr)TF_LPTR(stage + addr + (16 * s) * 512));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (LdsBf16x4Ptr)TF_LPTR(stage + addr + (16 * s + 4) * 512));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
        // chunk index 2 s + lhalf, swizzled: 2 s only touches bits 1..2 of the chunk, lhalf bit 0
        return *reinterpret_cast<const bf16x8*>(stage + (addr ^ (s << 5)));
    }
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
__global__ __launch_bounds__(kThreads) void gemm_mfma_kernel(GemmBatch batch) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];

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
    // byte advance of the global pointers per contraction step of 64
    const int64_t kstep_a = kTN ? int64_t(kBK) * lda * 2 : kBK * 2;
    const int64_t kstep_b = kTN ? int64_t(kBK) * ldb * 2 : kBK * 2;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const FillPtrs fp = make_fill<kTN>(A, B, lda, ldb, m0, n0);
    const FragAddr fr = make_frag_addr<kTN>(wm, wn);
    const int nk = Kc / kBK;

    // LDS byte address of the dynamic shared array (a 32-bit LDS pointer is its byte offset)
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        uint32_t(reinterpret_cast<uintptr_t>(TF_LPTR(lds))));
    fill_stage<kTN>(fp, 0, 0, lds_base);
    wait_direct_loads();
    __syncthreads();                      // this wave's loads have landed, now everyone else's too

    for (int kt = 0; kt < nk; ++kt) {
        const char* cur = lds + (kt & 1) * kStageBytes;
        const uint32_t nxt = lds_base + ((kt + 1) & 1) * kStageBytes;
        // The last step has nothing left to fetch; it re-fetches its own tile into the stage
        // nobody reads any more, which keeps the loop body one straight-line block.
        const int kn = min(kt + 1, nk - 1);
        const int64_t koff_a = kn * kstep_a, koff_b = kn * kstep_b;

        // Issue order is pinned with scheduling fences: operands of step 0, then every MFMA of
        // step s is followed by one operand read of step s + 1 and, in step 0, by one
        // direct-to-LDS load of the next stage, so LDS and memory latency hide behind the
        // matrix cores.
        bf16x8 fa[2][4], fb[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[0][i] = load_frag<kTN>(cur, fr.a[i], 0);
            fb[0][i] = load_frag<kTN>(cur, fr.b[i], 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < kBK / 16; ++s) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int i = q >> 2, j = q & 3;
                // D rows <- n (B operand rows), D columns <- m: a lane then owns 4 consecutive n
                // of one output row m, i.e. 4 contiguous elements of row-major C.
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
                if (s + 1 < kBK / 16 && q < 8) {
                    if (q & 1) fb[(s + 1) & 1][q >> 1] = load_frag<kTN>(cur, fr.b[q >> 1], s + 1);
                    else       fa[(s + 1) & 1][q >> 1] = load_frag<kTN>(cur, fr.a[q >> 1], s + 1);
                }
                if (s == 0) fill_one<kTN>(fp, koff_a, koff_b, nxt, q);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        wait_direct_loads();
        __syncthreads();                  // next stage landed everywhere, this one is free to overwrite
    }

    // epilogue: acc[i][j][4g + e] is C[m][n] with m = m0 + wm*128 + i*32 + lane%32,
    // n = n0 + wn*128 + j*32 + 8g + 4*(lane/32) + e.
    const int lrow = lane & 31, lhalf = lane >> 5;
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
