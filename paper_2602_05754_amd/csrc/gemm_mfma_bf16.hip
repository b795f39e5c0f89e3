// Grouped bf16 GEMM on the gfx950 matrix cores for the two halves of a backward
// action (TimelyFreeze Sec. 3.2.1):
//   kNT  dX = dY W^T   - contraction (N_l) is the contiguous index of both inputs
//   kTN  dW = X^T dY   - contraction (T) is the slow index of both inputs
// Only tensors that are not frozen are ever listed in a kTN batch, so a frozen
// tensor's dW tiles cost nothing and its buffers are never touched.
//
// One 256 x 256 output tile per workgroup.  The waves form a 2 x kWN grid
// (kWN = 2: 4 waves of 128 x 128, 256 accumulators per lane; kWN = 4: 8 waves of
// 128 x 64, 128 accumulators per lane, two waves per SIMD), each wave owning
// 4 x (8 / kWN) MFMA 32x32x16 tiles.  The contraction advances 64 at a time
// through two LDS stages of 64 KB that are filled by direct global->LDS loads
// (no register staging): while the matrix cores work on one stage the next one
// is in flight.  A stage is consumed in four steps of 16; the operands of step
// s + 1 are read from LDS while the MFMAs of step s issue, the stage barrier
// sits after the reads of the last step, and the first operands of the next
// stage are read during the last step, so neither LDS latency nor the barrier
// leaves the matrix cores idle.
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
constexpr int kTileBytes = kBM * kBK * 2;             // 32 KB per operand per stage
constexpr int kStageBytes = 2 * kTileBytes;           // A + B
constexpr int kLdsBytes = 2 * kStageBytes;            // two stages = 128 KB
constexpr int kGroupM = 8;                            // tile rows per L2 locality group
constexpr int kXcds = 8;
constexpr int kXcdRun = 32;                           // consecutive logical tiles kept on one XCD

#ifndef TF_GEMM_WN
#define TF_GEMM_WN 2
#endif

template <int kWN>
struct Shape {
    static constexpr int kWaves = 2 * kWN;                  // 4 or 8
    static constexpr int kThreads = 64 * kWaves;
    static constexpr int kWaveN = kBN / kWN;                // columns per wave: 128 or 64
    static constexpr int kNJ = kWaveN / 32;                 // MFMA column blocks per wave: 4 or 2
    static constexpr int kMfmaPerStep = 4 * kNJ;            // 16 or 8
    static constexpr int kReadsPerStep = 4 + kNJ;           // operand fragments per step: 8 or 6
    static constexpr int kLoadsPerOperand = 32 / kWaves;    // 1 KB loads per wave, operand and stage: 8 or 4
    static constexpr int kLoads = 2 * kLoadsPerOperand;     // 16 or 8
    // Loads of a stage fill issued in step 3 / in the next step 0 (the rest, if any, in step 1).
    // Half and half measured best; later loads arrive too late for the stage barrier.
    static constexpr int kLoadsStep3 = kLoads / 2;
    static constexpr int kLoadsStep0 = kLoads - kLoadsStep3;
    static constexpr int kEpiBytes = kLdsBytes / kWaves;    // LDS per wave for the epilogue: 32 or 16 KB
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));
typedef uint32_t U4 __attribute__((ext_vector_type(4)));
typedef float F4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4* LdsBf16x4Ptr;

#define TF_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// two binary32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
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
// Stage fill.  Load p of wave w fills KB number (p kWaves + w) of the 32 KB operand tile.
//   kNT: that KB is tile rows R = 8 (p kWaves + w) + lane/8, physical chunk lane%8 of each row;
//        logical chunk = physical ^ ((R ^ (R >> 3)) & 7).
//   kTN: that KB is contraction rows T = 2 (p kWaves + w) + lane/32, 16-byte slot lane%32 of
//        each; logical 64-byte block = physical block ^ (T & 3).
// ---------------------------------------------------------------------------------------------
struct FillPtrs {
    const char* base_a;       // wave-uniform global byte address of the tile's first element
    const char* base_b;
    int64_t pstep_a, pstep_b; // wave-uniform byte distance between loads p and p + 1
    uint32_t voff_a[2];       // per-lane byte offsets (even / odd p; they differ only for kNT with 4 waves)
    uint32_t voff_b[2];
};

template <bool kTN, int kWN>
__device__ __forceinline__ FillPtrs make_fill(const uint16_t* A, const uint16_t* B, int64_t lda, int64_t ldb,
                                              int m0, int n0) {
    constexpr int kWaves = Shape<kWN>::kWaves;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    FillPtrs f;
    if (kTN) {
        const int T = 2 * w + (lane >> 5);                     // + 2 kWaves p
        const int slot = lane & 31;
        const int blk = (slot >> 2) ^ (T & 3);
        const int col = blk * 32 + (slot & 3) * 8;             // element offset inside the 256-wide tile row
        f.base_a = reinterpret_cast<const char*>(A + m0);
        f.base_b = reinterpret_cast<const char*>(B + n0);
        f.voff_a[0] = f.voff_a[1] = uint32_t((int64_t(T) * lda + col) * 2);
        f.voff_b[0] = f.voff_b[1] = uint32_t((int64_t(T) * ldb + col) * 2);
        f.pstep_a = 2 * kWaves * lda * 2; f.pstep_b = 2 * kWaves * ldb * 2;
    } else {
        const int r = 8 * w + (lane >> 3);                     // + 8 kWaves p
        const int pc = lane & 7;
        f.base_a = reinterpret_cast<const char*>(A + int64_t(m0) * lda);
        f.base_b = reinterpret_cast<const char*>(B + int64_t(n0) * ldb);
#pragma unroll
        for (int q = 0; q < 2; ++q) {                          // p even / odd
            const int R = r + 8 * kWaves * q;
            const int c = pc ^ ((R ^ (R >> 3)) & 7);
            f.voff_a[q] = uint32_t((int64_t(r) * lda + c * 8) * 2);
            f.voff_b[q] = uint32_t((int64_t(r) * ldb + c * 8) * 2);
        }
        f.pstep_a = 8 * kWaves * lda * 2; f.pstep_b = 8 * kWaves * ldb * 2;
    }
    return f;
}

// One direct-to-LDS load: lane i fetches 16 bytes from gbase + voff and the wave's 1 KB lands
// at LDS byte address lds_wave_base + kLdsOff + 16 i (the LDS address goes through M0).
// Written as inline assembly so that the compiler's wait-count insertion does not treat every
// later LDS read as dependent on it (it would drain the load queue before each transpose read);
// completion is awaited explicitly with wait_direct_loads() before the stage barrier.
// The assembly must leave SCC alone: the compiler is free to place it between the two halves
// of one of its own 64-bit scalar additions (s_add_u32 / s_addc_u32), and a clobbered carry
// sends the high word of a global address off by one as soon as the addition crosses a
// 4 GiB boundary.  Hence s_mov_b32 for M0, with the LDS address added up outside.
template <int kLdsOff>
__device__ __forceinline__ void direct_load_16B(const char* gbase, uint32_t voff, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_wave_base + uint32_t(kLdsOff)), "v"(voff), "s"(gbase)
                 : "memory");
}
__device__ __forceinline__ void wait_direct_loads() {
    __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0), other counters untouched
}

// Issue load number q (0 .. kLoads-1) of a stage fill: even q fetch operand A, odd q operand B,
// load p = q / 2.  ka / kb are the wave-uniform byte offsets of the contraction step to fetch;
// lds_wave_base is the LDS byte address of the stage plus 1 KB times the wave index.
template <bool kTN, int kWN, int q>
__device__ __forceinline__ void fill_one(const FillPtrs& f, int64_t ka, int64_t kb, uint32_t lds_wave_base) {
    constexpr int p = q >> 1;
    constexpr int kOff = p * Shape<kWN>::kWaves * 1024;
    if ((q & 1) == 0) direct_load_16B<kOff>(f.base_a + ka + p * f.pstep_a, f.voff_a[p & 1], lds_wave_base);
    else direct_load_16B<kTileBytes + kOff>(f.base_b + kb + p * f.pstep_b, f.voff_b[p & 1], lds_wave_base);
}

template <bool kTN, int kWN, int q, int end>
__device__ __forceinline__ void fill_range(const FillPtrs& f, int64_t ka, int64_t kb, uint32_t lds_wave_base) {
    if constexpr (q < end) {
        fill_one<kTN, kWN, q>(f, ka, kb, lds_wave_base);
        fill_range<kTN, kWN, q + 1, end>(f, ka, kb, lds_wave_base);
    }
}

// Run-time index -> compile-time load number (the LDS offset of a load is an immediate).
template <bool kTN, int kWN>
__device__ __forceinline__ void fill_switch(int load, const FillPtrs& f, int64_t ka, int64_t kb, uint32_t dst) {
    switch (load) {
#define TF_FILL_CASE(Q) case Q: if constexpr (Q < Shape<kWN>::kLoads) fill_one<kTN, kWN, Q>(f, ka, kb, dst); break;
        TF_FILL_CASE(0) TF_FILL_CASE(1) TF_FILL_CASE(2) TF_FILL_CASE(3)
        TF_FILL_CASE(4) TF_FILL_CASE(5) TF_FILL_CASE(6) TF_FILL_CASE(7)
        TF_FILL_CASE(8) TF_FILL_CASE(9) TF_FILL_CASE(10) TF_FILL_CASE(11)
        TF_FILL_CASE(12) TF_FILL_CASE(13) TF_FILL_CASE(14) TF_FILL_CASE(15)
#undef TF_FILL_CASE
        default: break;
    }
}

// ---------------------------------------------------------------------------------------------
// MFMA operand fetch for contraction step s (16 values) of the current stage.
// Operand lane l holds row (l % 32) of a 32-row block and contraction values 8 (l / 32) .. + 7.
// ---------------------------------------------------------------------------------------------
template <int kWN>
struct FragAddr {
    int a[4], b[Shape<kWN>::kNJ];     // per-lane LDS byte offsets (inside a stage) of the row blocks, step 0
};

template <bool kTN, int kWN>
__device__ __forceinline__ FragAddr<kWN> make_frag_addr(int wm, int wn) {
    constexpr int kNJ = Shape<kWN>::kNJ, kWaveN = Shape<kWN>::kWaveN;
    const int lane = threadIdx.x & 63;
    FragAddr<kWN> fa;
    if (kTN) {
        // 16-lane group G reads rows 8 (G / 2) + {0..3} (+4 for the second read) of the
        // contraction and columns 16 (G % 2) + {0..15} of the 32-row block; as a source lane
        // ii of its group it fetches row ii / 4, columns 4 (ii % 4) .. + 3.
        const int G = lane >> 4, ii = lane & 15;
        const int x = ii >> 2;
        const int laneoff = (8 * (G >> 1) + x) * 512 + 32 * (G & 1) + 8 * (ii & 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) fa.a[i] = laneoff + (((wm * 4 + i) ^ x) * 64);
#pragma unroll
        for (int j = 0; j < kNJ; ++j) fa.b[j] = kTileBytes + laneoff + (((wn * kNJ + j) ^ x) * 64);
    } else {
        const int lrow = lane & 31, lhalf = lane >> 5;
        // chunk (2 s + lhalf) ^ swz(row): the s-dependent part is XORed in at use
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ra = wm * 128 + i * 32 + lrow;
            fa.a[i] = ra * 128 + ((lhalf ^ ((ra ^ (ra >> 3)) & 7)) << 4);
        }
#pragma unroll
        for (int j = 0; j < kNJ; ++j) {
            const int rb = wn * kWaveN + j * 32 + lrow;
            fa.b[j] = kTileBytes + rb * 128 + ((lhalf ^ ((rb ^ (rb >> 3)) & 7)) << 4);
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

template <bool kTN, bool kOutBf16, bool kAccumulate, int kWN>
__global__ __launch_bounds__(Shape<kWN>::kThreads) void gemm_mfma_kernel(GemmBatch batch) {
    using S = Shape<kWN>;
    constexpr int kNJ = S::kNJ;
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
    const int wm = wave / kWN, wn = wave % kWN;

    f32x16 acc[4][kNJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < kNJ; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const FillPtrs fp = make_fill<kTN, kWN>(A, B, lda, ldb, m0, n0);
    const FragAddr<kWN> fr = make_frag_addr<kTN, kWN>(wm, wn);
    const int nk = Kc / kBK;

    // LDS byte address of the dynamic shared array (a 32-bit LDS pointer is its byte offset),
    // plus this wave's 1 KB slot inside every group of kWaves KB of a stage fill.
    const uint32_t lds_wave_base = __builtin_amdgcn_readfirstlane(
        uint32_t(reinterpret_cast<uintptr_t>(TF_LPTR(lds))) + uint32_t(wave) * 1024u);

    // prologue: stage 0 <- step 0 completely, stage 1 <- first part of step 1 (the loop issues the rest)
    fill_range<kTN, kWN, 0, S::kLoads>(fp, 0, 0, lds_wave_base);
    wait_direct_loads();
    __syncthreads();
    {
        const int k1 = min(1, nk - 1);
        fill_range<kTN, kWN, 0, S::kLoadsStep3>(fp, k1 * kstep_a, k1 * kstep_b, lds_wave_base + kStageBytes);
    }
    bf16x8 fa[2][4], fb[2][kNJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[0][i] = load_frag<kTN>(lds, fr.a[i], 0);
#pragma unroll
    for (int j = 0; j < kNJ; ++j) fb[0][j] = load_frag<kTN>(lds, fr.b[j], 0);

    for (int kt = 0; kt < nk; ++kt) {
        const char* cur = lds + (kt & 1) * kStageBytes;
        const char* nxt = lds + ((kt + 1) & 1) * kStageBytes;
        const uint32_t cur_fill = lds_wave_base + (kt & 1) * kStageBytes;
        const uint32_t nxt_fill = lds_wave_base + ((kt + 1) & 1) * kStageBytes;
        // Contraction step fetched into `cur` once everybody is done reading it; past the end
        // the last step is fetched again (into a stage nobody reads any more), which keeps the
        // loop body free of branches.
        const int kf = min(kt + 2, nk - 1), kf1 = min(kt + 1, nk - 1);
        const int64_t ka = kf * kstep_a, kb = kf * kstep_b;          // fetched during step 3, into `cur`
        const int64_t ka1 = kf1 * kstep_a, kb1 = kf1 * kstep_b;      // rest of the previous fill, into `nxt`

        // Issue order below is pinned with scheduling fences.
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s == 3) {
                // every operand read of this stage has been issued: wait for them and for this
                // wave's part of the next stage, then meet the other waves.  After the barrier
                // the next stage is complete and this one may be overwritten.
                wait_direct_loads();
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            const char* rd = s == 3 ? nxt : cur;     // step 3 reads step 0 of the next stage
            const int rs = s == 3 ? 0 : s + 1;
#pragma unroll
            for (int q = 0; q < S::kMfmaPerStep; ++q) {
                const int i = q / kNJ, j = q % kNJ;
                // D rows <- n (B operand rows), D columns <- m: a lane then owns 4 consecutive n
                // of one output row m, i.e. 4 contiguous elements of row-major C.
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
                if (q < S::kReadsPerStep) {
                    // operand order A0 B0 A1 B1 ... then the remaining A blocks
                    if (q < 2 * kNJ) {
                        if (q & 1) fb[(s + 1) & 1][q >> 1] = load_frag<kTN>(rd, fr.b[q >> 1], rs);
                        else       fa[(s + 1) & 1][q >> 1] = load_frag<kTN>(rd, fr.a[q >> 1], rs);
                    } else {
                        fa[(s + 1) & 1][q - kNJ] = load_frag<kTN>(rd, fr.a[q - kNJ], rs);
                    }
                }
                // The loads of one stage fill are spread over step 3 (right after the barrier that
                // frees the stage) and steps 0 and 1 of the next stage's turn, so that the
                // texture-address unit, which the waves share, is never asked for more than it
                // can take while the matrix cores run.
                {
                    constexpr int n3 = S::kLoadsStep3, n0 = S::kLoadsStep0, n1 = S::kLoads - n3 - n0;
                    const int cnt = s == 3 ? n3 : s == 0 ? n0 : s == 1 ? n1 : 0;
                    const int first = s == 3 ? 0 : s == 0 ? n3 : n3 + n0;
                    if (cnt > 0) {
                        // spread `cnt` loads evenly over the MFMA slots of this step
                        const int before = (q * cnt) / S::kMfmaPerStep, after = ((q + 1) * cnt) / S::kMfmaPerStep;
                        if (after > before) {
                            if (s == 3) fill_switch<kTN, kWN>(first + before, fp, ka, kb, cur_fill);
                            else        fill_switch<kTN, kWN>(first + before, fp, ka1, kb1, nxt_fill);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    wait_direct_loads();      // nothing of this workgroup may still be in flight towards LDS

    // epilogue: acc[i][j][4g + e] is C[m][n] with m = m0 + wm*128 + i*32 + lane%32,
    // n = n0 + wn*kWaveN + j*32 + 8g + 4*(lane/32) + e.  A lane's values are scattered over the
    // tile, so each wave first turns its block around in its own share of the (now idle) LDS
    // and then writes whole rows.
    __syncthreads();                                   // every wave is done reading the stages
    char* wlds = lds + wave * S::kEpiBytes;
    const int lrow = lane & 31, lhalf = lane >> 5;
    constexpr int kChunks = S::kWaveN / 4;             // 4-element chunks per row of the wave's block: 32 or 16
    if (kOutBf16) {
        // [128 rows][kChunks chunks of 8 bytes]; the chunk index is XORed with a row number so
        // that the 32 rows written by one instruction fall into different banks
        constexpr int kPitch = S::kWaveN * 2;
        const int xw = kChunks == 32 ? lrow : (lrow >> 1);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < kNJ; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int m = i * 32 + lrow, c = 8 * j + 2 * g + lhalf;
                    *reinterpret_cast<U2*>(wlds + m * kPitch + ((c ^ xw) << 3)) =
                        U2{f32x2_to_bf16x2(acc[i][j][4 * g + 0], acc[i][j][4 * g + 1]),
                           f32x2_to_bf16x2(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3])};
                }
        constexpr int kLanesPerRow = kPitch / 16, kRowsPerInstr = 64 / kLanesPerRow;
        const int cb = lane % kLanesPerRow, rsub = lane / kLanesPerRow;   // 16-byte column block, row in group
        uint16_t* Cw = static_cast<uint16_t*>(P.C) + int64_t(m0 + wm * 128) * N + n0 + wn * S::kWaveN + cb * 8;
#pragma unroll 8
        for (int it = 0; it < 128 / kRowsPerInstr; ++it) {
            const int m = it * kRowsPerInstr + rsub;
            const int x = kChunks == 32 ? (m & 31) : ((m >> 1) & 15);
            // chunks 2cb and 2cb+1 sit in one aligned 16-byte pair, swapped when x is odd
            U4 v = *reinterpret_cast<const U4*>(wlds + m * kPitch + (((2 * cb) ^ (x & ~1)) << 3));
            if (x & 1) v = U4{v.z, v.w, v.x, v.y};
            *reinterpret_cast<U4*>(Cw + int64_t(m) * N) = v;
        }
    } else {
        // fp32: two passes of 64 rows, [64 rows][kChunks chunks of 16 bytes].  When accumulating,
        // the old values are fetched a batch of 16 row groups ahead (into registers the main loop
        // no longer needs), so that their HBM latency overlaps the LDS turn-around and the stores.
        constexpr int kPitch = S::kWaveN * 4;
        constexpr int kLanesPerRow = kPitch / 16, kRowsPerInstr = 64 / kLanesPerRow;
        constexpr int kIt = 64 / kRowsPerInstr;            // row groups per pass: 32 or 16
        constexpr int kBatch = 16, kBatchesPerPass = kIt / kBatch, kBatches = 2 * kBatchesPerPass;
        const int cb = lane % kLanesPerRow, rsub = lane / kLanesPerRow;
        float* Cw = static_cast<float*>(P.C) + int64_t(m0 + wm * 128) * N + n0 + wn * S::kWaveN + cb * 4;
        // row of the wave's block handled by row group `it` of batch `b`
        auto row_of = [&](int b, int it) { return (b / kBatchesPerPass) * 64 + ((b % kBatchesPerPass) * kBatch + it) * kRowsPerInstr + rsub; };
        F4 old[2][kBatch];
        auto fetch_old = [&](int b) {
#pragma unroll
            for (int it = 0; it < kBatch; ++it) old[b & 1][it] = *reinterpret_cast<const F4*>(Cw + int64_t(row_of(b, it)) * N);
        };
        if (kAccumulate) fetch_old(0);
#pragma unroll
        for (int b = 0; b < kBatches; ++b) {
            if (kAccumulate && b + 1 < kBatches) fetch_old(b + 1);
            if (b % kBatchesPerPass == 0) {
                const int h = b / kBatchesPerPass;
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < kNJ; ++j)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int i = 2 * h + ii;
                            const int m = ii * 32 + lrow, c = 8 * j + 2 * g + lhalf;
                            *reinterpret_cast<F4*>(wlds + m * kPitch + ((c ^ (lrow & (kChunks - 1))) << 4)) =
                                F4{acc[i][j][4 * g + 0], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        }
            }
#pragma unroll
            for (int it = 0; it < kBatch; ++it) {
                const int row = row_of(b, it), m = row & 63;
                F4 v = *reinterpret_cast<const F4*>(wlds + m * kPitch + ((cb ^ (m & (kChunks - 1))) << 4));
                if (kAccumulate) v += old[b & 1][it];
                *reinterpret_cast<F4*>(Cw + int64_t(row) * N) = v;
            }
        }
    }
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
hipError_t launch_one(hipStream_t stream, const GemmBatch& batch) {
    constexpr int kWN = TF_GEMM_WN;
    auto kern = gemm_mfma_kernel<kTN, kOutBf16, kAccumulate, kWN>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(batch.total_tiles), dim3(Shape<kWN>::kThreads), kLdsBytes, stream, batch);
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
