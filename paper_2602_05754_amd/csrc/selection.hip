// Device side of the metric-aware selection steps that sit next to the hot path.
//
// 1. AutoFreeze (TimelyFreeze Sec. 2.3): the score of a layer compares the norms of
//    its cumulative updates Delta_{K-1}, Delta_K between stability checks.  Delta_K is
//    p_now - p_at_the_previous_check, so one pass per check over the master weights
//    and a snapshot gives sum((p - snapshot)^2) per tensor and renews the snapshot.
//    HBM-bound: 8 B read + 4 B written per element; nothing is paid between checks.
//
// 2. Budget reconciliation of the hybrid variants (App. "Hybrid Variants Algorithm",
//    Alg. 2): a base element mask is brought to exactly N_freeze ones by adding
//    uniformly drawn zeros or removing uniformly drawn ones.  "Uniformly drawn" is made
//    reproducible by ranking candidates by the image of their stage-wide index under a
//    keyed permutation of [0, 2^32) (6-round Feistel network on 16-bit halves, round
//    function: top half of ((half ^ key) + 1) * 0x9E3779B1 mod 2^32) and taking the
//    lowest ranks.  The rank threshold is found by a radix select over the keys
//    (digits of 11, 11 and 10 bits): one histogram pass per digit and a one-thread
//    kernel that picks the bin, all on the stream - the host never waits.
//    ALU-bound: ~40 integer operations per candidate and pass, 1 bit of traffic.
#include "tf_internal.h"

namespace tf {
namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------------------------------
// AutoFreeze norms
// ------------------------------------------------------------------------------------------
// The launch shape follows the fused optimizer pass (what decides the rate is how the three
// streams meet in the memory system): a block is ONE wave and each of its accesses is 1 KB of one
// array (whole 128-byte lines); an unused 8 KB of dynamic LDS per block caps a compute unit at 20
// blocks; every access is non-temporal.  Measured on the 8B stage's 1.74e9 elements: 6.6 TB/s
// with 2 iterations per block and 20 blocks per unit (1 iteration: 5.4; 4: 6.5; 8: 5.9; 10 blocks
// per unit: 4.7 .. 6.1), against 5.5 for blocks of four waves and 8 iterations.
// With 3.4 million blocks the per-tensor sums are gathered in two levels like the optimizer's
// score sums: a block adds to one of 64 slots of its tensor, a second kernel adds up the slots.
constexpr int kNormThreads = 64;
constexpr int kNormGroup = 4, kNormIters = 2;
constexpr int kNormResidencyLds = 8192;
constexpr int kNormSlotDouble = 2;          // which double of a 64-byte slot (0 and 1 are the optimizer's)
constexpr int64_t kNormElemsPerBlock = int64_t(kNormThreads) * kNormGroup * kNormIters;
typedef float F4 __attribute__((ext_vector_type(4)));

// One wave per tensor: adds up the tensor's slots, writes the sum and leaves the slots zero for
// the next launch.
__global__ __launch_bounds__(kSumSlots) void norm_finish_kernel(NormBatch batch) {
    static_assert(kSumSlots == 64, "one wave reads one tensor's slots");
    double* slot = batch.partials + (int64_t(blockIdx.x) * kSumSlots + threadIdx.x) * kSumSlotDoubles + kNormSlotDouble;
    double x = *slot;
    *slot = 0.0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    if (threadIdx.x == 0) *batch.t[blockIdx.x].out = x;
}

__device__ __forceinline__ double block_sum(double x, double* lds4) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) lds4[wave] = x;
    __syncthreads();
    return lds4[0] + lds4[1] + lds4[2] + lds4[3];       // meaningful in every thread
}

__global__ __launch_bounds__(kNormThreads) void norm_kernel(NormBatch batch) {
    int ti = 0;
    const int bid = blockIdx.x;
    for (int i = 1; i < batch.n_tensors; ++i)
        if (bid >= batch.t[i].block_start) ti = i;
    const NormTensor& T = batch.t[ti];
    const int64_t numel = T.numel;
    const int local_block = bid - T.block_start;
    const int64_t chunk = int64_t(local_block) * kNormElemsPerBlock;
    double acc = 0.0;
#pragma unroll
    for (int it = 0; it < kNormIters; ++it) {
        const int64_t j = chunk + (int64_t(it) * kNormThreads + threadIdx.x) * kNormGroup;
        if (j + kNormGroup <= numel) {
            // streamed once: non-temporal accesses measured 5 % faster
            const F4 p = __builtin_nontemporal_load(reinterpret_cast<const F4*>(T.p + j));
            const F4 s = __builtin_nontemporal_load(reinterpret_cast<const F4*>(T.snap + j));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = double(p[e]) - double(s[e]);      // exact
                acc += d * d;
            }
            if (batch.update_snapshot) __builtin_nontemporal_store(p, reinterpret_cast<F4*>(T.snap + j));
        } else {
            for (int64_t q = j; q < numel; ++q) {                  // ragged tail
                const double d = double(T.p[q]) - double(T.snap[q]);
                acc += d * d;
                if (batch.update_snapshot) T.snap[q] = T.p[q];
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (threadIdx.x == 0)
        unsafeAtomicAdd(batch.partials + (int64_t(ti) * kSumSlots + local_block % kSumSlots) * kSumSlotDoubles + kNormSlotDouble, acc);
}

// ------------------------------------------------------------------------------------------
// Budget reconciliation
// ------------------------------------------------------------------------------------------
constexpr int kWordsPerThread = 4;
constexpr int kWordsPerBlock = kThreads * kWordsPerThread;          // 1024 words = 32768 elements
constexpr int kBins = 2048;

struct RcWord {
    uint32_t* ptr;        // the word, or nullptr past the end of the tensor
    uint32_t valid;       // bits of the word that are elements of the tensor
    uint32_t index0;      // stage-wide index of bit 0
};

__device__ __forceinline__ RcWord rc_word(const RcBatch& batch, int w) {
    int ti = 0;
    const int bid = blockIdx.x;
    for (int i = 1; i < batch.n_tensors; ++i)
        if (bid >= batch.t[i].block_start) ti = i;
    const RcTensor& T = batch.t[ti];
    const int64_t word = int64_t(bid - T.block_start) * kWordsPerBlock + int64_t(w) * kThreads + threadIdx.x;
    const int64_t n_words = (T.numel + 31) >> 5;
    RcWord r;
    if (word >= n_words) { r.ptr = nullptr; r.valid = 0; r.index0 = 0; return r; }
    const int64_t left = T.numel - (word << 5);
    r.ptr = T.bits + word;
    r.valid = left >= 32 ? 0xffffffffu : ((1u << int(left)) - 1u);
    r.index0 = uint32_t(T.goff + (word << 5));
    return r;
}

__global__ void rc_reset_kernel(RcState* st) {
    for (int i = threadIdx.x; i < kBins; i += blockDim.x) st->hist[i] = 0;
    if (threadIdx.x == 0) { st->count = 0; st->mode = 0; st->need = 0; st->prefix = 0; st->prefix_bits = 0; }
}

__global__ __launch_bounds__(kThreads) void rc_count_kernel(RcBatch batch, RcState* st) {
    __shared__ double part[4];
    uint32_t c = 0;
#pragma unroll
    for (int w = 0; w < kWordsPerThread; ++w) {
        const RcWord r = rc_word(batch, w);
        if (r.ptr) c += __popc(*r.ptr & r.valid);
    }
    const double total = block_sum(double(c), part);               // <= 32768 per block: exact
    if (threadIdx.x == 0 && total > 0.0) atomicAdd(&st->count, (unsigned long long)total);
}

// mode 0: the base mask already holds n_freeze ones; 1: add `need` of its zeros; 2: remove `need` of its ones
__global__ void rc_decide_kernel(RcState* st, unsigned long long n_freeze, long long* stats) {
    if (threadIdx.x != 0) return;
    const unsigned long long c = st->count;
    st->mode = c == n_freeze ? 0u : (c < n_freeze ? 1u : 2u);
    st->need = c < n_freeze ? n_freeze - c : c - n_freeze;
    st->prefix = 0; st->prefix_bits = 0;
    if (stats) { stats[0] = (long long)c; stats[1] = st->mode; stats[2] = 0; }
}

// Histogram of the digit (key >> shift) & (2^nbits - 1) over the candidates whose key starts with
// the prefix found so far.
__global__ __launch_bounds__(kThreads) void rc_hist_kernel(RcBatch batch, RcState* st, RcKeys keys, int shift, int nbits) {
    __shared__ uint32_t h[kBins];
    const uint32_t mode = st->mode;
    if (mode == 0) return;                                          // block-uniform
    for (int i = threadIdx.x; i < kBins; i += kThreads) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = st->prefix;
    const int pbits = int(st->prefix_bits);
    const uint32_t dmask = (1u << nbits) - 1u;
#pragma unroll 1
    for (int w = 0; w < kWordsPerThread; ++w) {
        const RcWord r = rc_word(batch, w);
        if (!r.ptr) continue;
        uint32_t cand = (mode == 1 ? ~*r.ptr : *r.ptr) & r.valid;
        while (cand) {
            const int b = __ffs(cand) - 1;
            cand &= cand - 1;
            const uint32_t key = perm32(r.index0 + uint32_t(b), keys);
            if (pbits == 0 || (key >> (32 - pbits)) == prefix) atomicAdd(&h[(key >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += kThreads)
        if (h[i]) atomicAdd(&st->hist[i], h[i]);
}

// Pick the bin in which the need-th smallest key lies; extend the prefix by its digit.
// One block of 256 threads: each sums 8 neighbouring bins, thread 0 walks the 256 partial sums
// and then the 8 bins of the one that holds the rank; all of them clear the histogram.
__global__ __launch_bounds__(kThreads) void rc_pick_kernel(RcState* st, int nbits, int last, long long* stats) {
    __shared__ unsigned long long part[kThreads];
    constexpr int kPer = kBins / kThreads;
    unsigned long long mine = 0;
    for (int q = 0; q < kPer; ++q) mine += st->hist[threadIdx.x * kPer + q];
    part[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0 && st->mode != 0) {
        const int bins = 1 << nbits;
        unsigned long long before = 0;
        int g = 0;
        for (; g < kThreads - 1 && (g + 1) * kPer < bins; ++g) {
            if (before + part[g] >= st->need) break;
            before += part[g];
        }
        int b = g * kPer;
        for (; b < bins - 1; ++b) {
            const unsigned long long hb = st->hist[b];
            if (before + hb >= st->need) break;
            before += hb;
        }
        st->need -= before;                      // rank inside the bin, >= 1
        st->prefix = (st->prefix << nbits) | uint32_t(b);
        st->prefix_bits += uint32_t(nbits);
        if (last && stats) stats[2] = (long long)st->prefix;
    }
    if (threadIdx.x == 0 && st->mode == 0 && last && stats) stats[2] = 0;
    __syncthreads();
    for (int q = 0; q < kPer; ++q) st->hist[threadIdx.x * kPer + q] = 0;
}

// After the last digit the prefix is a full key: the need-th smallest.  Candidates with a key
// not above it are the drawn ones.
__global__ __launch_bounds__(kThreads) void rc_apply_kernel(RcBatch batch, const RcState* st, RcKeys keys) {
    const uint32_t mode = st->mode;
    if (mode == 0) return;
    const uint32_t threshold = st->prefix;
#pragma unroll 1
    for (int w = 0; w < kWordsPerThread; ++w) {
        const RcWord r = rc_word(batch, w);
        if (!r.ptr) continue;
        const uint32_t old = *r.ptr;
        uint32_t cand = (mode == 1 ? ~old : old) & r.valid;
        uint32_t drawn = 0;
        while (cand) {
            const int b = __ffs(cand) - 1;
            cand &= cand - 1;
            if (perm32(r.index0 + uint32_t(b), keys) <= threshold) drawn |= 1u << b;
        }
        if (drawn) *r.ptr = mode == 1 ? (old | drawn) : (old & ~drawn);
    }
}

// grid: (chunks, runs).  Run blockIdx.y, words [blockIdx.x * 4096 ...) four per thread and sweep.
__global__ __launch_bounds__(kThreads) void fill_words_kernel(FillBatch batch) {
    const FillRunDesc& R = batch.r[blockIdx.y];
    for (int64_t w = int64_t(blockIdx.x) * kThreads + threadIdx.x; w < R.n_words; w += int64_t(gridDim.x) * kThreads)
        R.dst[w] = R.value;
}

}  // namespace

hipError_t launch_fill_words(hipStream_t stream, const FillBatch& batch) {
    if (batch.n_runs == 0) return hipSuccess;
    int64_t longest = 0;
    for (int i = 0; i < batch.n_runs; ++i) longest = batch.r[i].n_words > longest ? batch.r[i].n_words : longest;
    int64_t bx = (longest + kThreads * 4 - 1) / (kThreads * 4);
    if (bx < 1) bx = 1;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(fill_words_kernel, dim3(unsigned(bx), unsigned(batch.n_runs)), dim3(kThreads), 0, stream, batch);
    return hipGetLastError();
}

int64_t norm_elems_per_block() { return kNormElemsPerBlock; }
int64_t rc_elems_per_block() { return int64_t(kWordsPerBlock) * 32; }
size_t rc_state_bytes() { return sizeof(RcState); }

hipError_t launch_autofreeze_norms(hipStream_t stream, NormBatch& batch, int n_tensors, bool update_snapshot) {
    batch.n_tensors = n_tensors;
    batch.update_snapshot = update_snapshot ? 1 : 0;
    if (n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    if (!batch.partials) return hipErrorInvalidValue;
    hipLaunchKernelGGL(norm_kernel, dim3(batch.total_blocks), dim3(kNormThreads), kNormResidencyLds, stream, batch);
    hipLaunchKernelGGL(norm_finish_kernel, dim3(n_tensors), dim3(kSumSlots), 0, stream, batch);
    return hipGetLastError();
}

hipError_t launch_rc_begin(hipStream_t stream, RcState* st) {
    hipLaunchKernelGGL(rc_reset_kernel, dim3(1), dim3(256), 0, stream, st);
    return hipGetLastError();
}
hipError_t launch_rc_count(hipStream_t stream, RcBatch& batch, RcState* st) {
    if (batch.n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(rc_count_kernel, dim3(batch.total_blocks), dim3(kThreads), 0, stream, batch, st);
    return hipGetLastError();
}
hipError_t launch_rc_decide(hipStream_t stream, RcState* st, uint64_t n_freeze, int64_t* stats) {
    hipLaunchKernelGGL(rc_decide_kernel, dim3(1), dim3(64), 0, stream, st, (unsigned long long)n_freeze,
                       reinterpret_cast<long long*>(stats));
    return hipGetLastError();
}
hipError_t launch_rc_hist(hipStream_t stream, RcBatch& batch, RcState* st, const RcKeys& keys, int shift, int nbits) {
    if (batch.n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(rc_hist_kernel, dim3(batch.total_blocks), dim3(kThreads), 0, stream, batch, st, keys, shift, nbits);
    return hipGetLastError();
}
hipError_t launch_rc_pick(hipStream_t stream, RcState* st, int nbits, bool last, int64_t* stats) {
    hipLaunchKernelGGL(rc_pick_kernel, dim3(1), dim3(kThreads), 0, stream, st, nbits, last ? 1 : 0,
                       reinterpret_cast<long long*>(stats));
    return hipGetLastError();
}
hipError_t launch_rc_apply(hipStream_t stream, RcBatch& batch, RcState* st, const RcKeys& keys) {
    if (batch.n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(rc_apply_kernel, dim3(batch.total_blocks), dim3(kThreads), 0, stream, batch, st, keys);
    return hipGetLastError();
}

}  // namespace tf
