// Internal declarations shared by the translation units of libtf.so.
// Host-side launch functions; every one only enqueues on `stream`.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tf {

enum class Dtype : int { F32 = 0, BF16 = 1 };

// ---------------------------------------------------------------------------
// Grouped GEMM problem: C[M x N] (+)= sum_k A(m,k) * B(n,k), C row-major.
//   kNT ("rows share the contraction"): A is [M x Kc] row-major, B is [N x Kc]
//        row-major  ->  the input-gradient product dX = dY * W^T
//        (A = dY [T x N_l], B = W [K_l x N_l], C = dX [T x K_l]).
//   kTN ("contraction is the slow dimension"): A is [Kc x M] row-major, B is
//        [Kc x N] row-major  ->  the weight-gradient product dW = X^T * dY
//        (A = X [T x K_l], B = dY [T x N_l], C = dW [K_l x N_l]).
// ---------------------------------------------------------------------------
enum class Layout : int { kNT = 0, kTN = 1 };

struct GemmProblem {
    const void* A;
    const void* B;
    void* C;
    int32_t M, N, Kc;
    int32_t tile_start;     // first tile index of this problem inside a launch
    int32_t lda, ldb;       // row pitch of A and B in elements (kNT: >= Kc; kTN: >= M, >= N); C is dense
    // MFMA kernel only: which 256-row blocks of the output (and of A) exist.  Bit b set = block b is
    // computed; M counts the rows of the set bits only, tile row i of the problem is the i-th set
    // bit.  All ones = dense.  This is how frozen row blocks of a weight gradient are skipped
    // inside one grouped launch without touching their rows.
    uint64_t row_bits;
    // MFMA kernel only: the contraction of this problem continues over the next n_seg - 1 entries
    // of the batch (their A, B, Kc, lda, ldb; they own no tiles: tile_start = this problem's end).
    // C = sum over the segments of A_i B_i^T - several layers that share their input give ONE
    // input gradient, accumulated in fp32 and rounded once.  1 = an ordinary problem.
    int32_t n_seg;
    // MFMA kernel only, for a problem with fewer than 256 rows: operand rows that exist in memory
    // before row 0 (low 16 bits) and after row M - 1 (high 16 bits), each at most 256.  Its one
    // tile computes a 256-row window that runs over the problem's end or starts before its
    // beginning by that much, and stores only the problem's rows.  0 for M >= 256.
    uint32_t m_slack;
};

constexpr int kMaxProblemsPerLaunch = 64;

struct GemmBatch {          // passed by value as the kernel argument (64 x 64 B + 8 B = 4104 B)
    GemmProblem p[kMaxProblemsPerLaunch];
    int32_t n_problems;
    int32_t total_tiles;
};

// Edge-safe LDS-tiled FMA kernel (any M, N, Kc >= 1).  in: fp32 or bf16,
// accumulate fp32, out: fp32 (optionally +=) or bf16.
hipError_t launch_gemm_generic(hipStream_t stream, GemmBatch& batch, int n_problems,
                               Layout layout, Dtype in_dtype, Dtype out_dtype, bool accumulate);

// MFMA kernel for bf16 inputs.  What it takes (mfma_shape_ok): contraction a multiple of 64; output
// columns N >= 256 and a multiple of 8; output rows M >= 256, or fewer with rows_before +
// rows_after >= 256 - M operand rows in memory around them; layout kTN also M a multiple of 8; row
// pitches multiples of 8 and at most 2^22.  Extents need not be multiples of the 256 x 256 tile.
bool mfma_shape_ok(Layout layout, int64_t M, int64_t N, int64_t Kc, int64_t lda, int64_t ldb,
                   int64_t rows_before = 0, int64_t rows_after = 0);
hipError_t launch_gemm_mfma_bf16(hipStream_t stream, GemmBatch& batch, int n_problems,
                                 Layout layout, Dtype out_dtype, bool accumulate);
int gemm_generic_tile();          // tile edge of the generic kernel (square)
int gemm_mfma_tile();             // tile edge of the MFMA kernel (square)
int persistent_grid(int total_tiles, int units);    // workgroups of an MFMA launch on `units` compute units

// ---------------------------------------------------------------------------
// Fused elementwise pass: masked AdamW (+ APF EMAs) or the stand-alone EMA
// update.  One descriptor per unfrozen tensor.
// ---------------------------------------------------------------------------
struct EwTensor {
    float* p;               // fp32 master (adamw) / unused (stability)
    float* m;
    float* v;
    const void* g;          // gradient (adamw) or delta (stability, fp32)
    uint16_t* p_lowp;       // optional bf16 copy
    const uint32_t* bits;   // optional element mask, 1 = frozen
    float* E;               // optional (adamw) / required (stability)
    float* A;
    double* sums;           // optional: &score_sums[2*i]
    int64_t numel;
    float rbc1, rbc2;       // 1/(1-beta1^t), 1/(1-beta2^t)
};

constexpr int kMaxTensorsPerLaunch = 32;

// Per-tensor score sums are gathered in two levels: a block adds its two partial sums to one of
// kSumSlots slots of its tensor (one 64-byte line each, chosen by the block number), a second
// small kernel adds up the slots.  With one pair of addresses per tensor, the atomics of the
// 6.8 million one-wave blocks of the 8B stage would queue up behind each other (measured: 82 ms
// instead of 13).  The slots live in device memory owned by the context and are zero between launches.
constexpr int kSumSlots = 64;
constexpr int kSumSlotDoubles = 8;      // 64 bytes: {sum |E|, sum A, sum of squares of the AutoFreeze pass, unused...}
inline size_t ew_partials_bytes() { return size_t(kMaxTensorsPerLaunch) * kSumSlots * kSumSlotDoubles * sizeof(double); }

struct EwBatch {            // passed by value as the kernel argument (< 4 KB)
    EwTensor t[kMaxTensorsPerLaunch];
    int32_t block_start[kMaxTensorsPerLaunch];      // first block of each tensor inside the launch
    double* partials;       // the context's slots (device); needed only when some tensor wants sums
    int32_t n_tensors;
    int32_t total_blocks;
    // the caller's promise that every bf16 copy equals the rounding of its master weights on entry:
    // frozen elements of a partly frozen line then get their copy back from p instead of a re-read
    int32_t lowp_is_rounded_master;
    int32_t pad_;
};

struct AdamwParams {
    float grad_scale;
    float lr, beta1, beta2, eps, weight_decay;
    float one_minus_beta1, one_minus_beta2;
    float ema_decay, one_minus_ema_decay;
};

// ---------------------------------------------------------------------------
// AutoFreeze norms: out[i] = sum((p - snapshot)^2), snapshot <- p on request.
// ---------------------------------------------------------------------------
struct NormTensor {
    const float* p;
    float* snap;
    double* out;
    int64_t numel;
    int32_t block_start;
    int32_t pad_;
};
struct NormBatch {          // passed by value as the kernel argument
    NormTensor t[kMaxTensorsPerLaunch];
    double* partials;       // the context's slots (device), shared with the optimizer's score sums; zero between launches
    int32_t n_tensors;
    int32_t total_blocks;
    int32_t update_snapshot;
    int32_t pad_;
};
int64_t norm_elems_per_block();
hipError_t launch_autofreeze_norms(hipStream_t stream, NormBatch& batch, int n_tensors, bool update_snapshot);

// ---------------------------------------------------------------------------
// Budget reconciliation of an element mask (radix select over permutation keys).
// ---------------------------------------------------------------------------
struct RcTensor {
    uint32_t* bits;         // element mask, 1 = frozen, LSB first
    int64_t numel;
    int64_t goff;           // stage-wide index of element 0
    int32_t block_start;
    int32_t pad_;
};
struct RcBatch {            // passed by value as the kernel argument
    RcTensor t[kMaxTensorsPerLaunch];
    int32_t n_tensors;
    int32_t total_blocks;
};
struct RcKeys { uint32_t k[6]; };      // round keys of the index permutation

// Keyed permutation of [0, 2^32): 6-round Feistel network on 16-bit halves; round function:
// top 16 bits of ((half ^ key) + 1) * 0x9E3779B1 mod 2^32.
__host__ __device__ inline uint32_t perm32(uint32_t x, const RcKeys& k) {
    uint32_t hi = x >> 16, lo = x & 0xffffu;
    for (int r = 0; r < 6; ++r) {
        const uint32_t t = ((lo ^ k.k[r]) + 1u) * 0x9E3779B1u;
        const uint32_t nh = lo;
        lo = hi ^ (t >> 16);
        hi = nh;
    }
    return (hi << 16) | lo;
}
// Round keys: the four 16-bit pieces of the seed, low first, then bits 32..47 and 48..63 of
// seed * 0xD1342543DE82EF95 mod 2^64.
inline RcKeys perm32_keys(uint64_t seed) {
    RcKeys keys;
    const uint64_t s2 = seed * 0xD1342543DE82EF95ull;
    for (int r = 0; r < 4; ++r) keys.k[r] = uint32_t((seed >> (16 * r)) & 0xffffu);
    keys.k[4] = uint32_t((s2 >> 32) & 0xffffu);
    keys.k[5] = uint32_t((s2 >> 48) & 0xffffu);
    return keys;
}

// Fill runs of 32-bit words with a constant (element masks of whole row blocks).
struct FillRunDesc { uint32_t* dst; int64_t n_words; uint32_t value; uint32_t pad_; };
constexpr int kMaxFillRuns = 128;
struct FillBatch { FillRunDesc r[kMaxFillRuns]; int32_t n_runs; int32_t pad_; };
hipError_t launch_fill_words(hipStream_t stream, const FillBatch& batch);
struct RcState {            // device memory owned by the context
    uint32_t hist[2048];
    unsigned long long count;           // ones in the base mask
    unsigned long long need;            // rank still to be located
    uint32_t mode;                      // 0 keep, 1 add zeros, 2 remove ones
    uint32_t prefix, prefix_bits;       // leading key bits fixed so far
    uint32_t pad_;
};
int64_t rc_elems_per_block();
size_t rc_state_bytes();
hipError_t launch_rc_begin(hipStream_t stream, RcState* st);
hipError_t launch_rc_count(hipStream_t stream, RcBatch& batch, RcState* st);
hipError_t launch_rc_decide(hipStream_t stream, RcState* st, uint64_t n_freeze, int64_t* stats);
hipError_t launch_rc_hist(hipStream_t stream, RcBatch& batch, RcState* st, const RcKeys& keys, int shift, int nbits);
hipError_t launch_rc_pick(hipStream_t stream, RcState* st, int nbits, bool last, int64_t* stats);
hipError_t launch_rc_apply(hipStream_t stream, RcBatch& batch, RcState* st, const RcKeys& keys);

int64_t ew_elems_per_block();
hipError_t launch_adamw(hipStream_t stream, EwBatch& batch, int n_tensors,
                        const AdamwParams& hp, Dtype grad_dtype);
hipError_t launch_stability(hipStream_t stream, EwBatch& batch, int n_tensors,
                            const AdamwParams& hp);

}  // namespace tf
