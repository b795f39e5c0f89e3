// Fused masked AdamW + APF stability pass, and the stand-alone stability update.
//
// TimelyFreeze App. D.1: mask value 1 = frozen = no update (U = 1 - I); the
// optimizer is AdamW (Table exp_setup).  Sec. 2.3 (APF): E <- aE + (1-a)Delta,
// E^abs <- aE^abs + (1-a)|Delta|, with Delta = the update just applied.
//
// HBM-bound: per unfrozen element 22 B are read (p, m, v, E, A fp32 + bf16
// grad) and 22 B written (p, m, v, E, A + bf16 copy of p).  What decides the
// rate is how the twelve streams meet in the memory system, so the launch shape
// is chosen for that (measured, sustained, on the 8B stage's 1.74e9 elements):
//   * a block is ONE wave and covers 256 consecutive elements: each of its loads
//     and stores is 1 KB (0.5 KB for bf16) of one array, whole 128-byte lines;
//   * at most ten blocks are resident per compute unit (an unused 16 KB of
//     dynamic LDS per block caps it): with the full 32 waves per unit the same
//     code runs at 5.0 TB/s, with ten at 6.5 - fewer rows of DRAM open at once;
//   * every access is non-temporal: each byte is touched once.
// Element masks are applied per mask WORD = 32 elements = one 128-byte line of
// every fp32 array: a word that is all ones is skipped (nothing read, nothing
// written); any other word is processed as a whole, its frozen elements
// written back with the very bits that were read.  Skipping single 16-byte
// groups instead leaves partially written lines, which cost more than they
// save (3.5 TB/s at 70 % frozen elements).
#include "tf_internal.h"

namespace tf {
namespace {

constexpr int kThreads = 64;       // one wave
constexpr int kGroup = 4;          // consecutive elements per thread (one 16-byte fp32 vector)
constexpr int64_t kElemsPerBlock = int64_t(kThreads) * kGroup;        // 256 = 8 mask words
constexpr int kResidencyLds = 16384;   // bytes of dynamic LDS per block: 160 KB / 16 KB = 10 blocks per compute unit

typedef float F4 __attribute__((ext_vector_type(4)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// binary32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ void load4(const float* ptr, float (&out)[4]) {
    const F4 a = __builtin_nontemporal_load(reinterpret_cast<const F4*>(ptr));
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}

__device__ __forceinline__ void store4(float* ptr, const float (&in)[4]) {
    __builtin_nontemporal_store(F4{in[0], in[1], in[2], in[3]}, reinterpret_cast<F4*>(ptr));
}

// One element of the AdamW step; returns the applied update u = p_new - p_old.
__device__ __forceinline__ float adamw_elem(float& p, float& m, float& v, float g,
                                            const AdamwParams& hp, float rbc1, float rbc2) {
    m = hp.beta1 * m + hp.one_minus_beta1 * g;
    v = hp.beta2 * v + hp.one_minus_beta2 * (g * g);
    const float mhat = m * rbc1;
    const float vhat = v * rbc2;
    const float u = -(hp.lr * hp.weight_decay) * p - hp.lr * (mhat / (sqrtf(vhat) + hp.eps));
    p = p + u;
    return u;
}

__device__ __forceinline__ void ema_elem(float& E, float& A, float delta, const AdamwParams& hp) {
    E = hp.ema_decay * E + hp.one_minus_ema_decay * delta;
    A = hp.ema_decay * A + hp.one_minus_ema_decay * fabsf(delta);
}

// One block of kSumSlots threads per tensor: adds up the tensor's slots, writes the two sums and
// leaves the slots zero for the next launch.
__global__ __launch_bounds__(kSumSlots) void finish_sums_kernel(EwBatch batch) {
    static_assert(kSumSlots == 64, "one wave reads one tensor's slots");
    const EwTensor& T = batch.t[blockIdx.x];
    if (!T.sums) return;
    double* slot = batch.partials + (int64_t(blockIdx.x) * kSumSlots + threadIdx.x) * kSumSlotDoubles;
    double se = slot[0], sa = slot[1];
    slot[0] = 0.0; slot[1] = 0.0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        se += __shfl_down(se, off, 64);
        sa += __shfl_down(sa, off, 64);
    }
    if (threadIdx.x == 0) { T.sums[0] = se; T.sums[1] = sa; }
}

// kAdamw: full AdamW (+ EMAs if E != nullptr).  !kAdamw: EMAs from an explicit fp32 delta.
template <bool kAdamw, bool kGradBf16>
__global__ __launch_bounds__(kThreads) void ew_kernel(EwBatch batch, AdamwParams hp) {
    // locate this block's tensor: block-uniform scan over the 32 first-block numbers (entries past
    // n_tensors hold INT32_MAX), which sit together in the argument segment
    int ti = 0;
    const int bid = blockIdx.x;
#pragma unroll
    for (int i = 1; i < kMaxTensorsPerLaunch; ++i)
        if (bid >= batch.block_start[i]) ti = i;
    const EwTensor& T = batch.t[ti];
    const int64_t numel = T.numel;
    const int local_block = bid - batch.block_start[ti];
    const int64_t e0 = int64_t(local_block) * kElemsPerBlock + int64_t(threadIdx.x) * kGroup;
    const bool has_ema = T.E != nullptr;
    const bool want_sums = T.sums != nullptr;

    double sum_e = 0.0, sum_a = 0.0;

    if (e0 + kGroup <= numel) {
        // ---------------- vector path: 4 elements, the wave touches 1 KB of each fp32 array ----------------
        // the mask word of this group's line (8 lanes share it); its 4 bits for this group
        const uint32_t word = T.bits ? T.bits[e0 >> 5] : 0u;
        const uint32_t fz = (word >> (e0 & 28)) & 0xfu;
        if (word == 0xffffffffu) {
            // a wholly frozen line: untouched; its E, A still count in the sums
            if (want_sums) {
                float E[4], A[4];
                load4(T.E + e0, E);
                load4(T.A + e0, A);
                sum_e = double(fabsf(E[0]) + fabsf(E[1]) + fabsf(E[2]) + fabsf(E[3]));
                sum_a = double(A[0] + A[1] + A[2] + A[3]);
            }
        } else {
            float p[4], m[4], v[4], g[4], E[4], A[4];
            if (kAdamw) {
                load4(T.p + e0, p);
                load4(T.m + e0, m);
                load4(T.v + e0, v);
                if (kGradBf16) {
                    const U2 q = __builtin_nontemporal_load(reinterpret_cast<const U2*>(static_cast<const uint16_t*>(T.g) + e0));
                    g[0] = bf16_bits_to_f32(q.x & 0xffffu); g[1] = bf16_bits_to_f32(q.x >> 16);
                    g[2] = bf16_bits_to_f32(q.y & 0xffffu); g[3] = bf16_bits_to_f32(q.y >> 16);
                } else {
                    load4(static_cast<const float*>(T.g) + e0, g);
                }
            } else {
                load4(static_cast<const float*>(T.g) + e0, g);
            }
            if (has_ema) {
                load4(T.E + e0, E);
                load4(T.A + e0, A);
            }
            // The stored bf16 copy of frozen elements has to come back unchanged.  Unless the caller
            // has promised that the copy is the rounding of the master weights (then rounding the
            // unchanged p gives the same bits), it is read.
            U2 low_old = {0, 0};
            const bool has_low = kAdamw && T.p_lowp != nullptr;
            const bool reread_low = has_low && fz != 0u && !batch.lowp_is_rounded_master;
            if (reread_low) low_old = __builtin_nontemporal_load(reinterpret_cast<const U2*>(T.p_lowp + e0));

            uint32_t low[4];
            float se = 0.f, sa = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool frozen = (fz >> j) & 1u;
                float pn = 0.f, mn = 0.f, vn = 0.f, En = 0.f, An = 0.f;
                if (kAdamw) {
                    pn = p[j]; mn = m[j]; vn = v[j];
                    const float u = adamw_elem(pn, mn, vn, hp.grad_scale * g[j], hp, T.rbc1, T.rbc2);
                    if (has_ema) { En = E[j]; An = A[j]; ema_elem(En, An, u, hp); }
                    p[j] = frozen ? p[j] : pn;
                    m[j] = frozen ? m[j] : mn;
                    v[j] = frozen ? v[j] : vn;
                    low[j] = f32_to_bf16_bits(p[j]);
                } else {
                    En = E[j]; An = A[j]; ema_elem(En, An, g[j], hp);
                }
                if (has_ema) {
                    E[j] = frozen ? E[j] : En;
                    A[j] = frozen ? A[j] : An;
                    se += fabsf(E[j]); sa += A[j];
                }
            }
            if (kAdamw) {
                store4(T.p + e0, p);
                store4(T.m + e0, m);
                store4(T.v + e0, v);
                if (has_low) {
                    U2 o;
                    o.x = low[0] | (low[1] << 16); o.y = low[2] | (low[3] << 16);
                    if (reread_low) {
                        const uint32_t k0 = ((fz & 1u) ? 0xffffu : 0u) | ((fz & 2u) ? 0xffff0000u : 0u);
                        const uint32_t k1 = ((fz & 4u) ? 0xffffu : 0u) | ((fz & 8u) ? 0xffff0000u : 0u);
                        o.x = (o.x & ~k0) | (low_old.x & k0);
                        o.y = (o.y & ~k1) | (low_old.y & k1);
                    }
                    __builtin_nontemporal_store(o, reinterpret_cast<U2*>(T.p_lowp + e0));
                }
            }
            if (has_ema) {
                store4(T.E + e0, E);
                store4(T.A + e0, A);
                sum_e = double(se); sum_a = double(sa);
            }
        }
    } else if (e0 < numel) {
        // ---------------- ragged tail: < 4 elements, one at a time ----------------
        for (int64_t e = e0; e < numel; ++e) {
            const bool frozen = T.bits && ((T.bits[e >> 5] >> (e & 31)) & 1u);
            if (frozen) {
                if (want_sums) { sum_e += double(fabsf(T.E[e])); sum_a += double(T.A[e]); }
                continue;
            }
            float u;
            if (kAdamw) {
                float pn = T.p[e], mn = T.m[e], vn = T.v[e];
                float gj;
                if (kGradBf16) gj = bf16_bits_to_f32(static_cast<const uint16_t*>(T.g)[e]);
                else gj = static_cast<const float*>(T.g)[e];
                u = adamw_elem(pn, mn, vn, hp.grad_scale * gj, hp, T.rbc1, T.rbc2);
                T.p[e] = pn; T.m[e] = mn; T.v[e] = vn;
                if (T.p_lowp) T.p_lowp[e] = uint16_t(f32_to_bf16_bits(pn));
            } else {
                u = static_cast<const float*>(T.g)[e];
            }
            if (has_ema) {
                float En = T.E[e], An = T.A[e];
                ema_elem(En, An, u, hp);
                T.E[e] = En; T.A[e] = An;
                sum_e += double(fabsf(En)); sum_a += double(An);
            }
        }
    }

    if (want_sums) {
        // wave reduction (the block is one wave), then one fp64 atomic pair into one of the tensor's slots
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            sum_e += __shfl_down(sum_e, off, 64);
            sum_a += __shfl_down(sum_a, off, 64);
        }
        if (threadIdx.x == 0) {
            double* slot = batch.partials + (int64_t(ti) * kSumSlots + local_block % kSumSlots) * kSumSlotDoubles;
            unsafeAtomicAdd(slot + 0, sum_e);
            unsafeAtomicAdd(slot + 1, sum_a);
        }
    }
}

bool any_sums(const EwBatch& b, int n) {
    for (int i = 0; i < n; ++i)
        if (b.t[i].sums) return true;
    return false;
}

// Completes a batch whose first n_tensors descriptors and first-block numbers are filled in.
bool prepare(EwBatch& batch, int n_tensors) {
    batch.n_tensors = n_tensors;
    for (int i = n_tensors; i < kMaxTensorsPerLaunch; ++i) batch.block_start[i] = INT32_MAX;
    return !any_sums(batch, n_tensors) || batch.partials != nullptr;
}

}  // namespace

int64_t ew_elems_per_block() { return kElemsPerBlock; }

hipError_t launch_adamw(hipStream_t stream, EwBatch& batch, int n_tensors,
                        const AdamwParams& hp, Dtype grad_dtype) {
    if (!prepare(batch, n_tensors)) return hipErrorInvalidValue;
    if (n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    if (grad_dtype == Dtype::BF16)
        hipLaunchKernelGGL((ew_kernel<true, true>), dim3(batch.total_blocks), dim3(kThreads), kResidencyLds, stream, batch, hp);
    else
        hipLaunchKernelGGL((ew_kernel<true, false>), dim3(batch.total_blocks), dim3(kThreads), kResidencyLds, stream, batch, hp);
    if (any_sums(batch, n_tensors))
        hipLaunchKernelGGL(finish_sums_kernel, dim3(n_tensors), dim3(kSumSlots), 0, stream, batch);
    return hipGetLastError();
}

hipError_t launch_stability(hipStream_t stream, EwBatch& batch, int n_tensors,
                            const AdamwParams& hp) {
    if (!prepare(batch, n_tensors)) return hipErrorInvalidValue;
    if (n_tensors == 0 || batch.total_blocks == 0) return hipSuccess;
    hipLaunchKernelGGL((ew_kernel<false, false>), dim3(batch.total_blocks), dim3(kThreads), kResidencyLds, stream, batch, hp);
    if (any_sums(batch, n_tensors))
        hipLaunchKernelGGL(finish_sums_kernel, dim3(n_tensors), dim3(kSumSlots), 0, stream, batch);
    return hipGetLastError();
}

}  // namespace tf
