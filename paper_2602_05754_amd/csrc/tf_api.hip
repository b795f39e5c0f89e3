// C ABI of libtf.so: argument validation, host-side planning (which layers go
// into which grouped launch; frozen tensors are left out of the weight-gradient
// plan entirely) and kernel launches.  Declarations and contracts: include/tf.h.
#include "../../include/tf.h"
#include "tf_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

struct tf_prof_rec {
    int kind;
    hipEvent_t start, stop;
};

struct tf_ctx {
    int device_id;
    int last_hip_error;
    bool profiling;
    std::vector<tf_prof_rec> recs;      // events recorded since the last tf_profile_collect
    std::vector<hipEvent_t> pool;       // events ready for reuse
    tf::RcState* rc_state;              // device memory of tf_reconcile_mask (radix-select state)
    tf::RcState* rc_state_static;       // this device's static scratch array (tf_reconcile_mask_static)
    bool lowp_is_rounded_master;        // tf_assume_lowp_is_rounded_master
    double* ew_partials;                // device memory of the score sums' first level (zero between launches)
};

// Device memory of tf_reconcile_mask_static: one array per GPU, part of the loaded code object,
// alive until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returned for the current device.
constexpr size_t kStaticScratchBytes = 8448;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static_assert(sizeof(tf::RcState) <= kStaticScratchBytes, "the rank-search state must fit the static scratch array");

namespace {

using namespace tf;

constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices] = {nullptr};      // address of `scratch` on each device, set by tf_create

// With `device` current: the address of this device's copy of `scratch` (asked for once per device).
hipError_t static_scratch_address(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_addr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_addr[device] = ptr;
    }
    *out = g_scratch_addr[device];
    return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_dtype(int d) { return d == TF_F32 || d == TF_BF16; }
inline Dtype to_dtype(tf_dtype d) { return d == TF_BF16 ? Dtype::BF16 : Dtype::F32; }

int hip_fail(tf_ctx* ctx, hipError_t e) {
    ctx->last_hip_error = static_cast<int>(e);
    return TF_ERR_HIP;
}

// Optional per-kernel timing: a start/stop event pair around one launch, on the launch stream.
struct ProfScope {
    tf_ctx* ctx;
    hipStream_t stream;
    tf_prof_rec rec;
    bool on;
    ProfScope(tf_ctx* c, hipStream_t s, int kind) : ctx(c), stream(s), on(c->profiling) {
        if (!on) return;
        rec.kind = kind;
        for (hipEvent_t* e : {&rec.start, &rec.stop}) {
            if (!ctx->pool.empty()) { *e = ctx->pool.back(); ctx->pool.pop_back(); }
            else if (hipEventCreate(e) != hipSuccess) { on = false; return; }
        }
        (void)hipEventRecord(rec.start, stream);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(rec.stop, stream);
        ctx->recs.push_back(rec);
    }
};

// One planned GEMM: which layer, as which problem.
struct Planned {
    const void* A;
    const void* B;
    void* C;
    int64_t M, N, Kc;
    int64_t lda, ldb;       // row pitch of A, B in elements
    uint64_t row_bits;      // 256-row blocks that exist (MFMA kernel); all ones = dense
    // further contraction segments whose products are summed into the same C (layers that
    // share their input); matrix-core kernel only
    std::vector<Planned> more;
    int64_t rows_before = 0, rows_after = 0;   // operand rows in memory around the problem's own (sub-tensor problems)

    int64_t total_kc() const {
        int64_t k = Kc;
        for (const Planned& q : more) k += q.Kc;
        return k;
    }
};

inline bool planned_mfma_ok(const Planned& it, Layout layout, Dtype in_dtype) {
    return in_dtype == Dtype::BF16 && mfma_shape_ok(layout, it.M, it.N, it.Kc, it.lda, it.ldb, it.rows_before, it.rows_after) &&
           aligned16(it.A) && aligned16(it.B) && aligned16(it.C);
}

// Launch `items` in batches of at most kMaxProblemsPerLaunch, MFMA-eligible ones on the
// matrix cores, the rest on the generic kernel.
hipError_t launch_planned(tf_ctx* ctx, hipStream_t stream, std::vector<Planned>& items, Layout layout,
                          Dtype in_dtype, Dtype out_dtype, bool accumulate) {
    std::vector<Planned> fast, slow;
    for (const Planned& it : items) {
        bool ok = planned_mfma_ok(it, layout, in_dtype);
        for (const Planned& q : it.more) ok = ok && planned_mfma_ok(q, layout, in_dtype);
        if (ok) fast.push_back(it);
        else if (~it.row_bits != 0 || !it.more.empty()) return hipErrorInvalidValue;   // only the matrix-core kernel knows these
        else slow.push_back(it);
    }
    // Longest contraction first: the tail of a launch is then made of the cheapest tiles.
    auto by_cost = [](const Planned& a, const Planned& b) { return a.total_kc() > b.total_kc(); };
    std::stable_sort(fast.begin(), fast.end(), by_cost);
    std::stable_sort(slow.begin(), slow.end(), by_cost);

    GemmBatch batch;
    auto fill = [](GemmProblem& gp, const Planned& it, int64_t tile_start, int n_seg) {
        gp.A = it.A; gp.B = it.B; gp.C = it.C;
        gp.M = int32_t(it.M); gp.N = int32_t(it.N); gp.Kc = int32_t(it.Kc);
        gp.lda = int32_t(it.lda); gp.ldb = int32_t(it.ldb); gp.row_bits = it.row_bits;
        gp.tile_start = int32_t(tile_start);
        gp.n_seg = n_seg;
        // a problem narrower than one tile window: prefer running over its end to starting before its beginning
        const int64_t short_by = it.M < gemm_mfma_tile() ? gemm_mfma_tile() - it.M : 0;
        const int64_t after = std::min(it.rows_after, short_by), before = std::min(it.rows_before, short_by - after);
        gp.m_slack = uint32_t(before) | (uint32_t(after) << 16);
    };
    for (int pass = 0; pass < 2; ++pass) {
        const std::vector<Planned>& v = pass == 0 ? fast : slow;
        const int64_t tile = pass == 0 ? gemm_mfma_tile() : gemm_generic_tile();
        size_t i = 0;
        while (i < v.size()) {
            int n = 0;
            int64_t tiles = 0;
            while (i < v.size()) {
                const Planned& it = v[i];
                const int slots = 1 + int(it.more.size());
                if (slots > kMaxProblemsPerLaunch) return hipErrorInvalidValue;
                if (n + slots > kMaxProblemsPerLaunch) break;
                const int64_t nt = ((it.M + tile - 1) / tile) * ((it.N + tile - 1) / tile);
                if (nt > 0x3fffffff) return hipErrorInvalidValue;      // tile indices are 32-bit on the device
                if (n > 0 && tiles + nt > 0x3fffffff) break;
                fill(batch.p[n], it, tiles, slots);
                tiles += nt;
                ++n;
                for (const Planned& q : it.more) { fill(batch.p[n], q, tiles, 1); ++n; }     // own no tiles
                ++i;
            }
            batch.total_tiles = int32_t(tiles);
            const int kind = (layout == Layout::kNT ? TF_KERNEL_DX_MFMA : TF_KERNEL_DW_MFMA) + (pass == 0 ? 0 : 2);
            ProfScope prof(ctx, stream, kind);
            const hipError_t e = pass == 0
                ? launch_gemm_mfma_bf16(stream, batch, n, layout, out_dtype, accumulate)
                : launch_gemm_generic(stream, batch, n, layout, in_dtype, out_dtype, accumulate);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

// Byte ranges of a stage backward's tensors: an output may overlap neither an input nor
// another output (inputs may overlap each other).  Sweep over the ranges sorted by start.
struct ByteRange { uintptr_t lo, hi; bool output; };
bool outputs_overlap_something(std::vector<ByteRange>& r) {
    std::sort(r.begin(), r.end(), [](const ByteRange& a, const ByteRange& b) { return a.lo < b.lo; });
    uintptr_t end_any = 0, end_out = 0;          // furthest end among the ranges seen so far: all / outputs
    for (const ByteRange& x : r) {
        if (x.output ? x.lo < end_any : x.lo < end_out) return true;
        end_any = std::max(end_any, x.hi);
        if (x.output) end_out = std::max(end_out, x.hi);
    }
    return false;
}

// Later calls may come from another thread, or after the caller made another device current.
inline bool use_device(tf_ctx* ctx) {
    const hipError_t e = hipSetDevice(ctx->device_id);
    if (e != hipSuccess) { ctx->last_hip_error = static_cast<int>(e); return false; }
    return true;
}

int validate_elementwise_common(int32_t n_tensors, const int64_t* numel,
                                void* const* ema, void* const* ema_abs,
                                const uint8_t* tensor_freeze_mask,
                                const uint32_t* const* elem_freeze_bits,
                                const double* score_sums, float ema_decay, bool ema_required) {
    if (n_tensors < 0) return TF_ERR_INVALID_ARG;
    if (n_tensors == 0) return TF_OK;
    if (!numel) return TF_ERR_INVALID_ARG;
    if ((ema == nullptr) != (ema_abs == nullptr)) return TF_ERR_INVALID_ARG;
    if (ema_required && !ema) return TF_ERR_INVALID_ARG;
    if (score_sums && !ema) return TF_ERR_INVALID_ARG;
    if (ema && !(ema_decay >= 0.f && ema_decay <= 1.f)) return TF_ERR_INVALID_ARG;
    if (score_sums && (reinterpret_cast<uintptr_t>(score_sums) & 7u)) return TF_ERR_ALIGN;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (numel[i] <= 0) return TF_ERR_SHAPE;
        if (numel[i] > (int64_t(1) << 37)) return TF_ERR_SHAPE;      // 2^29 blocks of 256 elements per launch
        if (tensor_freeze_mask && tensor_freeze_mask[i] > 1) return TF_ERR_INVALID_ARG;
        if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
        if (ema) {
            if (!ema[i] || !ema_abs[i]) return TF_ERR_INVALID_ARG;
            if (!aligned16(ema[i]) || !aligned16(ema_abs[i])) return TF_ERR_ALIGN;
        }
        if (elem_freeze_bits && elem_freeze_bits[i] && !aligned16(elem_freeze_bits[i])) return TF_ERR_ALIGN;
    }
    return TF_OK;
}

// The stage backward behind every entry point.  `accumulate_mask`, when given, says layer by
// layer whether the weight gradient is added to dW_l (1) or overwrites it (0) and replaces
// `accumulate`.
int stage_backward_impl(tf_ctx* ctx, void* hip_stream,
                        int32_t n_layers, const tf_shape* shapes,
                        int64_t T, tf_dtype io_dtype,
                        const void* const* W, const void* const* X, const void* const* dY,
                        const uint8_t* freeze_mask,
                        const uint8_t* const* row_block_mask, int32_t block_rows,
                        const int32_t* input_group,
                        void* const* dX,
                        void* const* dW, tf_dtype dw_dtype,
                        int accumulate, const uint8_t* accumulate_mask) {
    // ---- validation: no HIP call before this block has passed ----
    if (n_layers < 0) return TF_ERR_INVALID_ARG;
    if (!valid_dtype(io_dtype) || !valid_dtype(dw_dtype)) return TF_ERR_DTYPE;
    if (accumulate != 0 && accumulate != 1) return TF_ERR_INVALID_ARG;
    if (accumulate_mask) {
        accumulate = 0;
        for (int32_t l = 0; l < n_layers; ++l) {
            if (accumulate_mask[l] > 1) return TF_ERR_INVALID_ARG;
            if (accumulate_mask[l] && !(freeze_mask && freeze_mask[l] == 1)) accumulate = 1;
        }
    }
    if (accumulate && dw_dtype != TF_F32) return TF_ERR_DTYPE;
    if (io_dtype == TF_F32 && dw_dtype != TF_F32) return TF_ERR_DTYPE;
    if (row_block_mask && block_rows <= 0) return TF_ERR_INVALID_ARG;
    if (n_layers > 0) {
        if (!shapes || !W || !dY || !dX) return TF_ERR_INVALID_ARG;
        if (T <= 0 || T > 0x7fffffff) return TF_ERR_SHAPE;
        bool any_unfrozen = false;
        for (int32_t l = 0; l < n_layers; ++l) {
            if (shapes[l].K <= 0 || shapes[l].N <= 0) return TF_ERR_SHAPE;
            if (shapes[l].K > 0x7fffffff || shapes[l].N > 0x7fffffff) return TF_ERR_SHAPE;
            if (freeze_mask && freeze_mask[l] > 1) return TF_ERR_INVALID_ARG;
            if (!W[l] || !dY[l] || !dX[l]) return TF_ERR_INVALID_ARG;
            if (!aligned16(W[l]) || !aligned16(dY[l]) || !aligned16(dX[l])) return TF_ERR_ALIGN;
            if (!(freeze_mask && freeze_mask[l])) any_unfrozen = true;
        }
        if (any_unfrozen && (!X || !dW)) return TF_ERR_INVALID_ARG;
        if (input_group) {
            // members of a group share their input: same K, same dX buffer; the first member leads
            for (int32_t l = 0; l < n_layers; ++l) {
                const int32_t g = input_group[l];
                if (g < -1 || g >= n_layers) return TF_ERR_INVALID_ARG;
                if (g < 0) continue;
                int32_t lead = l;
                for (int32_t q = 0; q < l; ++q) if (input_group[q] == g) { lead = q; break; }
                if (shapes[lead].K != shapes[l].K) return TF_ERR_SHAPE;
                if (dX[lead] != dX[l]) return TF_ERR_INVALID_ARG;
            }
        }
        for (int32_t l = 0; l < n_layers; ++l) {
            if (freeze_mask && freeze_mask[l]) continue;
            if (!X[l] || !dW[l]) return TF_ERR_INVALID_ARG;
            if (!aligned16(X[l]) || !aligned16(dW[l])) return TF_ERR_ALIGN;
            if (row_block_mask && row_block_mask[l]) {
                if (shapes[l].K % block_rows != 0) return TF_ERR_SHAPE;
                for (int64_t b = 0; b < shapes[l].K / block_rows; ++b)
                    if (row_block_mask[l][b] > 1) return TF_ERR_INVALID_ARG;
            }
        }
    }
    const int64_t in_size = io_dtype == TF_BF16 ? 2 : 4, dw_size = dw_dtype == TF_BF16 ? 2 : 4;
    if (n_layers > 0) {
        // no output may overlap an input or another output (the members of an input group pass
        // one dX buffer: it is listed once, for the member that leads the group)
        std::vector<ByteRange> ranges;
        ranges.reserve(size_t(n_layers) * 5);
        auto add = [&](const void* p, int64_t elems, int64_t size, bool output) {
            const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
            ranges.push_back(ByteRange{lo, lo + uintptr_t(elems) * uintptr_t(size), output});
        };
        std::vector<uint8_t> group_seen(input_group ? n_layers : 0, 0);
        for (int32_t l = 0; l < n_layers; ++l) {
            const int64_t K = shapes[l].K, N = shapes[l].N;
            add(W[l], K * N, in_size, false);
            add(dY[l], T * N, in_size, false);
            const int32_t g = input_group ? input_group[l] : -1;
            if (g < 0 || !group_seen[g]) add(dX[l], T * K, in_size, true);
            if (g >= 0) group_seen[g] = 1;
            if (freeze_mask && freeze_mask[l]) continue;
            add(X[l], T * K, in_size, false);
            add(dW[l], K * N, dw_size, true);
        }
        if (outputs_overlap_something(ranges)) return TF_ERR_ALIAS;
    }
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (n_layers == 0) return TF_OK;
    if (!use_device(ctx)) return TF_ERR_HIP;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Dtype in_dt = to_dtype(io_dtype);

    // input gradients: every layer, whatever the masks say.  Layers that share their input are
    // segments of one problem: their products are summed in the accumulators and rounded once.
    std::vector<Planned> plan;
    plan.reserve(n_layers);
    bool grouped_slow = false;
    {
        std::vector<int32_t> lead_slot(n_layers, -1);          // group id -> index in plan
        for (int32_t l = 0; l < n_layers; ++l) {
            Planned it{dY[l], W[l], dX[l], T, shapes[l].K, shapes[l].N, shapes[l].N, shapes[l].N, ~0ull, {}};
            const int32_t g = input_group ? input_group[l] : -1;
            if (g >= 0 && lead_slot[g] >= 0) plan[lead_slot[g]].more.push_back(it);
            else { if (g >= 0) lead_slot[g] = int32_t(plan.size()); plan.push_back(it); }
        }
        for (const Planned& it : plan) {
            if (it.more.empty()) continue;
            bool ok = planned_mfma_ok(it, Layout::kNT, in_dt);
            for (const Planned& q : it.more) ok = ok && planned_mfma_ok(q, Layout::kNT, in_dt);
            if (!ok) grouped_slow = true;
        }
    }
    hipError_t e = hipSuccess;
    if (!grouped_slow) {
        e = launch_planned(ctx, stream, plan, Layout::kNT, in_dt, in_dt, false);
    } else {
        // A group that the matrix-core kernel cannot take: member after member, each launch adding
        // onto the one before.  That needs an fp32 output (the fp32 configuration).
        if (in_dt != Dtype::F32) return TF_ERR_SHAPE;
        size_t depth = 0;
        for (const Planned& it : plan) depth = std::max(depth, it.more.size());
        for (size_t k = 0; k <= depth && e == hipSuccess; ++k) {
            std::vector<Planned> round;
            for (const Planned& it : plan) {
                if (k == 0) { Planned h = it; h.more.clear(); round.push_back(h); }
                else if (k <= it.more.size()) round.push_back(it.more[k - 1]);
            }
            e = launch_planned(ctx, stream, round, Layout::kNT, in_dt, in_dt, k > 0);
        }
    }
    if (e != hipSuccess) return hip_fail(ctx, e);

    // weight gradients: what is frozen - a layer, or a block of rows of one - is simply not
    // in the plan.
    // Layers whose gradient is added to what dW_l holds and layers whose gradient overwrites it
    // are two plans (two kernels: the adding one fetches the old values).
    plan.clear();
    std::vector<Planned> plan_set, plan_add;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (freeze_mask && freeze_mask[l]) continue;
        const bool add = accumulate_mask ? accumulate_mask[l] != 0 : accumulate != 0;
        std::vector<Planned>& dst = add ? plan_add : plan_set;
        const int64_t K = shapes[l].K, N = shapes[l].N;
        const uint8_t* rm = row_block_mask ? row_block_mask[l] : nullptr;
        if (!rm) {
            dst.push_back(Planned{X[l], dY[l], dW[l], K, N, T, K, N, ~0ull, {}});
            continue;
        }
        const int64_t nb = K / block_rows;
        // Matrix-core path: one problem per tensor whose tile rows are the unfrozen 256-row
        // blocks (a bit per block), so that any pattern of frozen blocks costs one problem.
        const int64_t tile = gemm_mfma_tile();
        if (in_dt == Dtype::BF16 && block_rows % tile == 0 && K / tile <= 64 &&
            mfma_shape_ok(Layout::kTN, tile, N, T, K, N) && aligned16(X[l]) && aligned16(dY[l]) && aligned16(dW[l])) {
            uint64_t bits = 0;
            int64_t rows = 0;
            const int64_t per = block_rows / tile;
            for (int64_t b = 0; b < nb; ++b)
                if (!rm[b])
                    for (int64_t q = 0; q < per; ++q) { bits |= 1ull << (b * per + q); rows += tile; }
            if (rows > 0) dst.push_back(Planned{X[l], dY[l], dW[l], rows, N, T, K, N, rows == K ? ~0ull : bits, {}});
            continue;
        }
        // Otherwise each run of unfrozen row blocks is one problem: columns [k0, k1) of X
        // (pitch K_l) against dY give rows [k0, k1) of dW.
        for (int64_t b = 0; b < nb;) {
            if (rm[b]) { ++b; continue; }
            int64_t e1 = b;
            while (e1 < nb && !rm[e1]) ++e1;
            const int64_t k0 = b * block_rows, rows = (e1 - b) * block_rows;
            Planned run{static_cast<const char*>(X[l]) + k0 * in_size, dY[l],
                        static_cast<char*>(dW[l]) + k0 * N * dw_size, rows, N, T, K, N, ~0ull, {}};
            run.rows_before = k0;                    // columns of X on either side of the run's own
            run.rows_after = K - k0 - rows;
            dst.push_back(run);
            b = e1;
        }
    }
    e = launch_planned(ctx, stream, plan_set, Layout::kTN, in_dt, to_dtype(dw_dtype), false);
    if (e != hipSuccess) return hip_fail(ctx, e);
    e = launch_planned(ctx, stream, plan_add, Layout::kTN, in_dt, to_dtype(dw_dtype), true);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return TF_OK;
}


}  // namespace

extern "C" {

const char* tf_version(void) { return "0.1.0"; }

const char* tf_strerror(int code) {
    switch (code) {
        case TF_OK: return "ok";
        case TF_ERR_INVALID_ARG: return "invalid argument";
        case TF_ERR_SHAPE: return "invalid shape or size";
        case TF_ERR_DTYPE: return "unsupported dtype or dtype combination";
        case TF_ERR_ALIGN: return "device pointer is not 16-byte aligned";
        case TF_ERR_WORKSPACE: return "workspace allocation failed";
        case TF_ERR_HIP: return "HIP runtime error (see tf_last_hip_error)";
        case TF_ERR_NO_DEVICE: return "no usable gfx950 device";
        case TF_ERR_ALIAS: return "an output buffer overlaps an input or another output";
        default: return "unknown status code";
    }
}

int tf_create(tf_ctx** out, int device_id) {
    if (!out || device_id < 0) return TF_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device_id >= count) return TF_ERR_NO_DEVICE;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device_id) != hipSuccess) return TF_ERR_NO_DEVICE;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return TF_ERR_NO_DEVICE;
    if (hipSetDevice(device_id) != hipSuccess) return TF_ERR_NO_DEVICE;
    tf_ctx* ctx = new (std::nothrow) tf_ctx;
    if (!ctx) return TF_ERR_WORKSPACE;
    ctx->device_id = device_id;
    ctx->last_hip_error = 0;
    ctx->profiling = false;
    ctx->rc_state = nullptr;
    ctx->rc_state_static = nullptr;
    ctx->lowp_is_rounded_master = false;
    ctx->ew_partials = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&ctx->rc_state), tf::rc_state_bytes()) != hipSuccess) {
        delete ctx;
        return TF_ERR_WORKSPACE;
    }
    void* st = nullptr;
    if (static_scratch_address(device_id, &st) != hipSuccess ||      // device_id is current here
        hipMalloc(reinterpret_cast<void**>(&ctx->ew_partials), tf::ew_partials_bytes()) != hipSuccess ||
        hipMemset(ctx->ew_partials, 0, tf::ew_partials_bytes()) != hipSuccess) {
        if (ctx->ew_partials) (void)hipFree(ctx->ew_partials);
        (void)hipFree(ctx->rc_state);
        delete ctx;
        return TF_ERR_WORKSPACE;
    }
    ctx->rc_state_static = static_cast<tf::RcState*>(st);
    *out = ctx;
    return TF_OK;
}

int tf_destroy(tf_ctx* ctx) {
    if (!ctx) return TF_ERR_INVALID_ARG;
    for (tf_prof_rec& r : ctx->recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (hipEvent_t e : ctx->pool) (void)hipEventDestroy(e);
    if (ctx->rc_state) (void)hipFree(ctx->rc_state);
    if (ctx->ew_partials) (void)hipFree(ctx->ew_partials);
    delete ctx;
    return TF_OK;
}

int tf_assume_lowp_is_rounded_master(tf_ctx* ctx, int on) {
    if (!ctx || (on != 0 && on != 1)) return TF_ERR_INVALID_ARG;
    ctx->lowp_is_rounded_master = on != 0;
    return TF_OK;
}

int tf_profile_enable(tf_ctx* ctx, int enable) {
    if (!ctx || (enable != 0 && enable != 1)) return TF_ERR_INVALID_ARG;
    ctx->profiling = enable != 0;
    return TF_OK;
}

int tf_profile_collect(tf_ctx* ctx, int32_t capacity, int32_t* kinds, float* ms, int32_t* n_out) {
    if (!ctx || !n_out || capacity < 0 || (capacity > 0 && (!kinds || !ms))) return TF_ERR_INVALID_ARG;
    int32_t n = 0;
    int rc = TF_OK;
    for (tf_prof_rec& r : ctx->recs) {
        if (n < capacity && rc == TF_OK) {
            hipError_t e = hipEventSynchronize(r.stop);
            float t = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
            if (e != hipSuccess) rc = hip_fail(ctx, e);
            else { kinds[n] = r.kind; ms[n] = t; ++n; }
        }
        ctx->pool.push_back(r.start);
        ctx->pool.push_back(r.stop);
    }
    ctx->recs.clear();
    *n_out = n;
    return rc;
}

int tf_last_hip_error(const tf_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

int tf_stage_backward_shared(tf_ctx* ctx, void* hip_stream,
                             int32_t n_layers, const tf_shape* shapes,
                             int64_t T, tf_dtype io_dtype,
                             const void* const* W, const void* const* X, const void* const* dY,
                             const uint8_t* freeze_mask,
                             const uint8_t* const* row_block_mask, int32_t block_rows,
                             const int32_t* input_group,
                             void* const* dX,
                             void* const* dW, tf_dtype dw_dtype,
                             int accumulate) {
    return stage_backward_impl(ctx, hip_stream, n_layers, shapes, T, io_dtype, W, X, dY, freeze_mask,
                               row_block_mask, block_rows, input_group, dX, dW, dw_dtype, accumulate, nullptr);
}

int tf_stage_backward_microbatch(tf_ctx* ctx, void* hip_stream,
                                 int32_t n_layers, const tf_shape* shapes,
                                 int64_t T, tf_dtype io_dtype,
                                 const void* const* W, const void* const* X, const void* const* dY,
                                 const uint8_t* freeze_mask,
                                 void* const* dX,
                                 void* const* dW, tf_dtype dw_dtype,
                                 const uint8_t* accumulate_mask) {
    if (n_layers > 0 && !accumulate_mask) return TF_ERR_INVALID_ARG;
    return stage_backward_impl(ctx, hip_stream, n_layers, shapes, T, io_dtype, W, X, dY, freeze_mask,
                               nullptr, 0, nullptr, dX, dW, dw_dtype, 0, accumulate_mask);
}

int tf_stage_backward(tf_ctx* ctx, void* hip_stream,
                      int32_t n_layers, const tf_shape* shapes,
                      int64_t T, tf_dtype io_dtype,
                      const void* const* W, const void* const* X, const void* const* dY,
                      const uint8_t* freeze_mask,
                      void* const* dX,
                      void* const* dW, tf_dtype dw_dtype,
                      int accumulate) {
    return tf_stage_backward_shared(ctx, hip_stream, n_layers, shapes, T, io_dtype, W, X, dY, freeze_mask,
                                    nullptr, 0, nullptr, dX, dW, dw_dtype, accumulate);
}

int tf_stage_backward_blocks(tf_ctx* ctx, void* hip_stream,
                             int32_t n_layers, const tf_shape* shapes,
                             int64_t T, tf_dtype io_dtype,
                             const void* const* W, const void* const* X, const void* const* dY,
                             const uint8_t* freeze_mask,
                             const uint8_t* const* row_block_mask, int32_t block_rows,
                             void* const* dX,
                             void* const* dW, tf_dtype dw_dtype,
                             int accumulate) {
    return tf_stage_backward_shared(ctx, hip_stream, n_layers, shapes, T, io_dtype, W, X, dY, freeze_mask,
                                    row_block_mask, block_rows, nullptr, dX, dW, dw_dtype, accumulate);
}

int tf_masked_adamw(tf_ctx* ctx, void* hip_stream,
                    int32_t n_tensors, const int64_t* numel,
                    void* const* p_master, void* const* m, void* const* v,
                    const void* const* grad, tf_dtype grad_dtype, float grad_scale,
                    void* const* p_lowp,
                    const uint8_t* tensor_freeze_mask,
                    const uint32_t* const* elem_freeze_bits,
                    const int32_t* step,
                    float lr, float beta1, float beta2, float eps, float weight_decay,
                    void* const* ema, void* const* ema_abs, float ema_decay,
                    double* score_sums) {
    if (!valid_dtype(grad_dtype)) return TF_ERR_DTYPE;
    int rc = validate_elementwise_common(n_tensors, numel, ema, ema_abs, tensor_freeze_mask,
                                         elem_freeze_bits, score_sums, ema_decay, false);
    if (rc != TF_OK) return rc;
    if (n_tensors > 0) {
        if (!p_master || !m || !v || !grad || !step) return TF_ERR_INVALID_ARG;
        if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return TF_ERR_INVALID_ARG;
        if (!(eps >= 0.f) || !std::isfinite(lr) || !std::isfinite(weight_decay) || !std::isfinite(grad_scale))
            return TF_ERR_INVALID_ARG;
        for (int32_t i = 0; i < n_tensors; ++i) {
            if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
            if (step[i] < 1) return TF_ERR_INVALID_ARG;
            if (!p_master[i] || !m[i] || !v[i] || !grad[i]) return TF_ERR_INVALID_ARG;
            if (!aligned16(p_master[i]) || !aligned16(m[i]) || !aligned16(v[i]) || !aligned16(grad[i]))
                return TF_ERR_ALIGN;
            if (p_lowp && p_lowp[i] && !aligned16(p_lowp[i])) return TF_ERR_ALIGN;
        }
    }
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (n_tensors == 0) return TF_OK;
    if (!use_device(ctx)) return TF_ERR_HIP;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    AdamwParams hp;
    hp.grad_scale = grad_scale;
    hp.lr = lr; hp.beta1 = beta1; hp.beta2 = beta2; hp.eps = eps; hp.weight_decay = weight_decay;
    hp.one_minus_beta1 = float(1.0 - double(beta1));
    hp.one_minus_beta2 = float(1.0 - double(beta2));
    hp.ema_decay = ema_decay;
    hp.one_minus_ema_decay = float(1.0 - double(ema_decay));

    const int64_t epb = ew_elems_per_block();
    EwBatch batch;
    batch.lowp_is_rounded_master = ctx->lowp_is_rounded_master ? 1 : 0;
    batch.pad_ = 0;
    batch.partials = ctx->ew_partials;
    int n = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> hipError_t {
        batch.total_blocks = int32_t(blocks);
        ProfScope prof(ctx, stream, TF_KERNEL_ADAMW);
        const hipError_t e = launch_adamw(stream, batch, n, hp, to_dtype(grad_dtype));
        n = 0; blocks = 0;
        return e;
    };
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;   // frozen: not even read
        const int64_t nb = (numel[i] + epb - 1) / epb;
        if (n == kMaxTensorsPerLaunch || (n > 0 && blocks + nb > 0x3fffffff)) {
            const hipError_t e = flush();
            if (e != hipSuccess) return hip_fail(ctx, e);
        }
        EwTensor& t = batch.t[n];
        t.p = static_cast<float*>(p_master[i]);
        t.m = static_cast<float*>(m[i]);
        t.v = static_cast<float*>(v[i]);
        t.g = grad[i];
        t.p_lowp = p_lowp ? static_cast<uint16_t*>(p_lowp[i]) : nullptr;
        t.bits = elem_freeze_bits ? elem_freeze_bits[i] : nullptr;
        t.E = ema ? static_cast<float*>(ema[i]) : nullptr;
        t.A = ema ? static_cast<float*>(ema_abs[i]) : nullptr;
        t.sums = score_sums ? score_sums + 2 * int64_t(i) : nullptr;
        t.numel = numel[i];
        t.rbc1 = float(1.0 / (1.0 - std::pow(double(beta1), double(step[i]))));
        t.rbc2 = float(1.0 / (1.0 - std::pow(double(beta2), double(step[i]))));
        batch.block_start[n] = int32_t(blocks);
        blocks += nb;
        ++n;
    }
    if (n > 0) {
        const hipError_t e = flush();
        if (e != hipSuccess) return hip_fail(ctx, e);
    }
    return TF_OK;
}

int tf_stability_update(tf_ctx* ctx, void* hip_stream,
                        int32_t n_tensors, const int64_t* numel,
                        const void* const* delta,
                        void* const* ema, void* const* ema_abs, float ema_decay,
                        const uint8_t* tensor_freeze_mask,
                        const uint32_t* const* elem_freeze_bits,
                        double* score_sums) {
    int rc = validate_elementwise_common(n_tensors, numel, ema, ema_abs, tensor_freeze_mask,
                                         elem_freeze_bits, score_sums, ema_decay, true);
    if (rc != TF_OK) return rc;
    if (n_tensors > 0) {
        if (!delta) return TF_ERR_INVALID_ARG;
        for (int32_t i = 0; i < n_tensors; ++i) {
            if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
            if (!delta[i]) return TF_ERR_INVALID_ARG;
            if (!aligned16(delta[i])) return TF_ERR_ALIGN;
        }
    }
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (n_tensors == 0) return TF_OK;
    if (!use_device(ctx)) return TF_ERR_HIP;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    AdamwParams hp;
    std::memset(&hp, 0, sizeof(hp));
    hp.ema_decay = ema_decay;
    hp.one_minus_ema_decay = float(1.0 - double(ema_decay));

    const int64_t epb = ew_elems_per_block();
    EwBatch batch;
    batch.lowp_is_rounded_master = 0;
    batch.pad_ = 0;
    batch.partials = ctx->ew_partials;
    int n = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> hipError_t {
        batch.total_blocks = int32_t(blocks);
        ProfScope prof(ctx, stream, TF_KERNEL_STABILITY);
        const hipError_t e = launch_stability(stream, batch, n, hp);
        n = 0; blocks = 0;
        return e;
    };
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
        const int64_t nb = (numel[i] + epb - 1) / epb;
        if (n == kMaxTensorsPerLaunch || (n > 0 && blocks + nb > 0x3fffffff)) {
            const hipError_t e = flush();
            if (e != hipSuccess) return hip_fail(ctx, e);
        }
        EwTensor& t = batch.t[n];
        std::memset(&t, 0, sizeof(t));
        t.g = delta[i];
        t.bits = elem_freeze_bits ? elem_freeze_bits[i] : nullptr;
        t.E = static_cast<float*>(ema[i]);
        t.A = static_cast<float*>(ema_abs[i]);
        t.sums = score_sums ? score_sums + 2 * int64_t(i) : nullptr;
        t.numel = numel[i];
        batch.block_start[n] = int32_t(blocks);
        blocks += nb;
        ++n;
    }
    if (n > 0) {
        const hipError_t e = flush();
        if (e != hipSuccess) return hip_fail(ctx, e);
    }
    return TF_OK;
}

int tf_stability_scores(const double* score_sums, int32_t n, double* scores) {
    if (n < 0 || (n > 0 && (!score_sums || !scores))) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        const double se = score_sums[2 * i], sa = score_sums[2 * i + 1];
        scores[i] = (sa == 0.0) ? 1.0 : se / sa;
    }
    return TF_OK;
}

int tf_select_lowest(const double* scores, int32_t n, int32_t n_freeze, uint8_t* out_mask) {
    if (n < 0 || n_freeze < 0 || n_freeze > n) return TF_ERR_INVALID_ARG;
    if (n > 0 && (!scores || !out_mask)) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (std::isnan(scores[i])) return TF_ERR_INVALID_ARG;
    std::vector<int32_t> order(n);
    for (int32_t i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return scores[a] < scores[b]; });
    for (int32_t i = 0; i < n; ++i) out_mask[i] = 0;
    for (int32_t i = 0; i < n_freeze; ++i) out_mask[order[i]] = 1;
    return TF_OK;
}

int tf_microbatch_plan(int32_t n_microbatches, int32_t n_layers, const uint8_t* freeze_masks,
                       uint8_t* accumulate_masks, uint8_t* step_freeze_mask) {
    if (n_microbatches < 0 || n_layers < 0) return TF_ERR_INVALID_ARG;
    if (n_layers == 0) return TF_OK;
    if (!step_freeze_mask || (n_microbatches > 0 && (!freeze_masks || !accumulate_masks))) return TF_ERR_INVALID_ARG;
    for (int64_t i = 0; i < int64_t(n_microbatches) * n_layers; ++i)
        if (freeze_masks[i] > 1) return TF_ERR_INVALID_ARG;
    for (int32_t l = 0; l < n_layers; ++l) {
        uint8_t seen = 0;                       // unfrozen in an earlier microbatch
        for (int32_t m = 0; m < n_microbatches; ++m) {
            accumulate_masks[int64_t(m) * n_layers + l] = seen;
            if (!freeze_masks[int64_t(m) * n_layers + l]) seen = 1;
        }
        step_freeze_mask[l] = seen ? 0 : 1;
    }
    return TF_OK;
}

int32_t tf_num_frozen(double r, int32_t n) {
    if (n <= 0 || !(r > 0.0)) return 0;
    const double x = std::ceil(r * double(n) - 1e-9);
    if (x >= double(n)) return n;
    return x < 0.0 ? 0 : int32_t(x);
}

int tf_autofreeze_norms(tf_ctx* ctx, void* hip_stream,
                        int32_t n_tensors, const int64_t* numel,
                        const void* const* p_master, void* const* snapshot,
                        const uint8_t* tensor_freeze_mask, int update_snapshot,
                        double* sq_norms) {
    if (n_tensors < 0 || (update_snapshot != 0 && update_snapshot != 1)) return TF_ERR_INVALID_ARG;
    if (n_tensors > 0) {
        if (!numel || !p_master || !snapshot || !sq_norms) return TF_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(sq_norms) & 7u) return TF_ERR_ALIGN;
        for (int32_t i = 0; i < n_tensors; ++i) {
            if (numel[i] <= 0 || numel[i] > (int64_t(1) << 40)) return TF_ERR_SHAPE;
            if (tensor_freeze_mask && tensor_freeze_mask[i] > 1) return TF_ERR_INVALID_ARG;
            if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
            if (!p_master[i] || !snapshot[i]) return TF_ERR_INVALID_ARG;
            if (!aligned16(p_master[i]) || !aligned16(snapshot[i])) return TF_ERR_ALIGN;
        }
    }
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (n_tensors == 0) return TF_OK;
    if (!use_device(ctx)) return TF_ERR_HIP;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t epb = norm_elems_per_block();
    NormBatch batch;
    batch.partials = ctx->ew_partials;
    int n = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> hipError_t {
        if (n == 0) return hipSuccess;
        batch.total_blocks = int32_t(blocks);
        ProfScope prof(ctx, stream, TF_KERNEL_AUTOFREEZE);
        const hipError_t e = launch_autofreeze_norms(stream, batch, n, update_snapshot != 0);
        n = 0; blocks = 0;
        return e;
    };
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (tensor_freeze_mask && tensor_freeze_mask[i]) continue;
        const int64_t nb = (numel[i] + epb - 1) / epb;
        if (n == kMaxTensorsPerLaunch || blocks + nb > 0x3fffffff) {
            const hipError_t e = flush();
            if (e != hipSuccess) return hip_fail(ctx, e);
        }
        NormTensor& t = batch.t[n];
        t.p = static_cast<const float*>(p_master[i]);
        t.snap = static_cast<float*>(snapshot[i]);
        t.out = sq_norms + i;
        t.numel = numel[i];
        t.block_start = int32_t(blocks);
        t.pad_ = 0;
        blocks += nb;
        ++n;
    }
    const hipError_t e = flush();
    if (e != hipSuccess) return hip_fail(ctx, e);
    return TF_OK;
}

int tf_autofreeze_scores(const double* sq_prev, const double* sq_cur, int32_t n, double* scores) {
    if (n < 0 || (n > 0 && (!sq_prev || !sq_cur || !scores))) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (!(sq_prev[i] >= 0.0) || !(sq_cur[i] >= 0.0)) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        const double a = std::sqrt(sq_prev[i]), b = std::sqrt(sq_cur[i]);
        if (a == 0.0) scores[i] = b == 0.0 ? 0.0 : INFINITY;
        else scores[i] = std::fabs(a - b) / a;
    }
    return TF_OK;
}

int tf_autofreeze_select(const double* scores, int32_t n, int32_t n_already_frozen,
                         double percentile, uint8_t* out_mask) {
    if (n < 0 || n_already_frozen < 0 || n_already_frozen > n) return TF_ERR_INVALID_ARG;
    if (!(percentile >= 0.0 && percentile <= 100.0)) return TF_ERR_INVALID_ARG;
    if (n > 0 && (!scores || !out_mask)) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (std::isnan(scores[i])) return TF_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) out_mask[i] = i < n_already_frozen ? 1 : 0;
    const int32_t n_active = n - n_already_frozen;
    if (n_active == 0) return TF_OK;
    std::vector<double> active(scores + n_already_frozen, scores + n);
    std::sort(active.begin(), active.end());
    const int32_t rank = int32_t(std::ceil(percentile / 100.0 * double(n_active) - 1e-9));
    if (rank <= 0) return TF_OK;
    const double tau = active[std::min(rank, n_active) - 1];
    for (int32_t l = n_already_frozen; l < n && scores[l] <= tau; ++l) out_mask[l] = 1;
    return TF_OK;
}

// Validation shared by the two reconciliation entry points (no HIP call).
static int validate_reconcile(int32_t n_tensors, const int64_t* numel, uint32_t* const* elem_bits,
                              int64_t n_freeze, const int64_t* stats) {
    if (n_tensors < 0 || n_freeze < 0) return TF_ERR_INVALID_ARG;
    if (n_tensors > 0 && (!numel || !elem_bits)) return TF_ERR_INVALID_ARG;
    if (stats && (reinterpret_cast<uintptr_t>(stats) & 7u)) return TF_ERR_ALIGN;
    int64_t total = 0;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (numel[i] <= 0) return TF_ERR_SHAPE;
        total += numel[i];
        if (total >= (int64_t(1) << 32)) return TF_ERR_SHAPE;
        if (!elem_bits[i]) return TF_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(elem_bits[i]) & 3u) return TF_ERR_ALIGN;
    }
    if (n_freeze > total) return TF_ERR_INVALID_ARG;
    return TF_OK;
}

// The passes of the reconciliation on the state `st`.  Allocates nothing, on the host or on the
// device: the tensor descriptors of a launch are built on the stack, pass after pass.
static hipError_t reconcile_passes(hipStream_t stream, int32_t n_tensors, const int64_t* numel,
                                   uint32_t* const* elem_bits, int64_t n_freeze, uint64_t seed,
                                   int64_t* stats, RcState* st) {
    const RcKeys keys = perm32_keys(seed);
    const int64_t epb = rc_elems_per_block();
    // calls fn(batch) for every launch-sized group of tensors, in order
    auto for_each_batch = [&](auto&& fn) -> hipError_t {
        RcBatch b;
        b.n_tensors = 0; b.total_blocks = 0;
        int64_t goff = 0, blocks = 0;
        for (int32_t i = 0; i < n_tensors; ++i) {
            const int64_t nb = (numel[i] + epb - 1) / epb;
            if (b.n_tensors == kMaxTensorsPerLaunch || blocks + nb > 0x3fffffff) {
                b.total_blocks = int32_t(blocks);
                const hipError_t e = fn(b);
                if (e != hipSuccess) return e;
                b.n_tensors = 0; blocks = 0;
            }
            RcTensor& t = b.t[b.n_tensors++];
            t.bits = elem_bits[i]; t.numel = numel[i]; t.goff = goff;
            t.block_start = int32_t(blocks); t.pad_ = 0;
            blocks += nb;
            goff += numel[i];
        }
        if (b.n_tensors > 0) { b.total_blocks = int32_t(blocks); return fn(b); }
        return hipSuccess;
    };
    hipError_t e = launch_rc_begin(stream, st);               // a kernel clears the state: nothing survives from the call before
    if (e == hipSuccess) e = for_each_batch([&](RcBatch& b) { return launch_rc_count(stream, b, st); });
    if (e == hipSuccess) e = launch_rc_decide(stream, st, uint64_t(n_freeze), stats);
    const int shifts[3] = {21, 10, 0}, widths[3] = {11, 11, 10};
    for (int pass = 0; pass < 3; ++pass) {
        if (e == hipSuccess) e = for_each_batch([&](RcBatch& b) { return launch_rc_hist(stream, b, st, keys, shifts[pass], widths[pass]); });
        if (e == hipSuccess) e = launch_rc_pick(stream, st, widths[pass], pass == 2, stats);
    }
    if (e == hipSuccess) e = for_each_batch([&](RcBatch& b) { return launch_rc_apply(stream, b, st, keys); });
    return e;
}

int tf_reconcile_mask(tf_ctx* ctx, void* hip_stream,
                      int32_t n_tensors, const int64_t* numel,
                      uint32_t* const* elem_bits,
                      int64_t n_freeze, uint64_t seed,
                      int64_t* stats) {
    const int rc = validate_reconcile(n_tensors, numel, elem_bits, n_freeze, stats);
    if (rc != TF_OK) return rc;
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (!use_device(ctx)) return TF_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    ProfScope prof(ctx, stream, TF_KERNEL_RECONCILE);
    const hipError_t e = reconcile_passes(stream, n_tensors, numel, elem_bits, n_freeze, seed, stats, ctx->rc_state);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return TF_OK;
}

int tf_reconcile_mask_static(tf_ctx* ctx, void* hip_stream,
                             int32_t n_tensors, const int64_t* numel,
                             uint32_t* const* elem_bits,
                             int64_t n_freeze, uint64_t seed,
                             int64_t* stats) {
    const int rc = validate_reconcile(n_tensors, numel, elem_bits, n_freeze, stats);     // sizes beyond 2^32 - 1 elements: TF_ERR_SHAPE
    if (rc != TF_OK) return rc;
    if (!ctx || !ctx->rc_state_static) return TF_ERR_INVALID_ARG;
    if (!use_device(ctx)) return TF_ERR_HIP;
    // no timing events here: creating one allocates
    const hipError_t e = reconcile_passes(static_cast<hipStream_t>(hip_stream), n_tensors, numel, elem_bits, n_freeze,
                                          seed, stats, ctx->rc_state_static);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return TF_OK;
}

int tf_select_row_blocks(int32_t n_layers, const tf_shape* shapes, int32_t block_rows,
                         double r, uint64_t seed, uint8_t* masks, int64_t* frozen_params) {
    if (n_layers < 0 || block_rows <= 0 || !(r >= 0.0 && r <= 1.0)) return TF_ERR_INVALID_ARG;
    if (n_layers > 0 && (!shapes || !masks)) return TF_ERR_INVALID_ARG;
    struct Unit { uint32_t key; int64_t size; int64_t pos; };
    std::vector<Unit> units;
    const RcKeys keys = perm32_keys(seed);
    int64_t total = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (shapes[l].K <= 0 || shapes[l].N <= 0 || shapes[l].K % block_rows != 0) return TF_ERR_SHAPE;
        for (int64_t b = 0; b < shapes[l].K / block_rows; ++b) {
            if (units.size() >= 0xffffffffull) return TF_ERR_SHAPE;
            const int64_t pos = int64_t(units.size());
            units.push_back(Unit{perm32(uint32_t(pos), keys), int64_t(block_rows) * shapes[l].N, pos});
            total += units.back().size;
        }
    }
    const int64_t budget = int64_t(std::floor(r * double(total) + 1e-9));
    std::sort(units.begin(), units.end(), [](const Unit& a, const Unit& b) { return a.key < b.key; });
    for (size_t i = 0; i < units.size(); ++i) masks[i] = 0;
    int64_t frozen = 0;
    for (const Unit& u : units)
        if (frozen + u.size <= budget) { frozen += u.size; masks[u.pos] = 1; }
    if (frozen_params) *frozen_params = frozen;
    return TF_OK;
}

int tf_row_blocks_to_bits(tf_ctx* ctx, void* hip_stream,
                          int32_t n_layers, const tf_shape* shapes,
                          const uint8_t* const* row_block_mask, int32_t block_rows,
                          uint32_t* const* elem_bits) {
    if (n_layers < 0 || block_rows <= 0) return TF_ERR_INVALID_ARG;
    if (n_layers > 0 && (!shapes || !elem_bits)) return TF_ERR_INVALID_ARG;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (shapes[l].K <= 0 || shapes[l].N <= 0) return TF_ERR_SHAPE;
        if (!elem_bits[l]) return TF_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(elem_bits[l]) & 3u) return TF_ERR_ALIGN;
        const uint8_t* rm = row_block_mask ? row_block_mask[l] : nullptr;
        if (rm) {
            if (shapes[l].K % block_rows != 0) return TF_ERR_SHAPE;
            if ((int64_t(block_rows) * shapes[l].N) % 32 != 0) return TF_ERR_SHAPE;     // blocks must end on word boundaries
            for (int64_t b = 0; b < shapes[l].K / block_rows; ++b)
                if (rm[b] > 1) return TF_ERR_INVALID_ARG;
        }
    }
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (!use_device(ctx)) return TF_ERR_HIP;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    FillBatch batch;
    batch.n_runs = 0; batch.pad_ = 0;
    auto push = [&](uint32_t* dst, int64_t n_words, uint32_t value) -> hipError_t {
        if (n_words <= 0) return hipSuccess;
        FillRunDesc& d = batch.r[batch.n_runs++];
        d.dst = dst; d.n_words = n_words; d.value = value; d.pad_ = 0;
        if (batch.n_runs == kMaxFillRuns) {
            const hipError_t e = launch_fill_words(stream, batch);
            batch.n_runs = 0;
            return e;
        }
        return hipSuccess;
    };
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t numel = shapes[l].K * shapes[l].N;
        const uint8_t* rm = row_block_mask ? row_block_mask[l] : nullptr;
        hipError_t e = hipSuccess;
        if (!rm) {
            e = push(elem_bits[l], (numel + 31) / 32, 0u);
        } else {
            const int64_t nb = shapes[l].K / block_rows, wpb = int64_t(block_rows) * shapes[l].N / 32;
            for (int64_t b = 0; b < nb && e == hipSuccess;) {
                int64_t e1 = b;
                while (e1 < nb && rm[e1] == rm[b]) ++e1;
                e = push(elem_bits[l] + b * wpb, (e1 - b) * wpb, rm[b] ? 0xffffffffu : 0u);
                b = e1;
            }
        }
        if (e != hipSuccess) return hip_fail(ctx, e);
    }
    const hipError_t e = launch_fill_words(stream, batch);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return TF_OK;
}

}  // extern "C"
