// Grouped bf16 GEMM on the gfx950 matrix cores for the two halves of a backward
// action (TimelyFreeze Sec. 3.2.1):
//   kNT  dX = dY W^T   - contraction (N_l) is the contiguous index of both inputs
//   kTN  dW = X^T dY   - contraction (T) is the slow index of both inputs
// Only tensors that are not frozen are ever listed in a kTN batch, so a frozen
// tensor's dW tiles cost nothing and its buffers are never touched.
//
// Persistent workgroups: one per compute unit, each walking every gridDim.x-th
// 256 x 256 output tile of the launch.  Four waves in a 2 x 2 grid, 128 x 128 per
// wave = 8 x 8 MFMA 16x16x32 tiles, 256 accumulators per lane.  The contraction
// advances 64 at a time through LDS stages of 32 KB per operand - two for A, three
// for B, all of the 160 KB - that are filled by direct global->LDS loads (no
// register staging): A's loads are issued one contraction step before they are
// awaited, B's 1 3/4 steps.  The fills form ONE stream over all tiles of the
// workgroup: while the matrix cores finish a tile, the first two contraction steps
// of the next tile are already in flight, so a tile switch costs the epilogue and
// nothing else - no drain, no refill, no new workgroup.
// A stage is consumed in two sub-steps of 32 (64 MFMAs each); the operands of the
// next sub-step are read from LDS while the MFMAs of this one issue, the stage
// barrier sits after the last reads of the stage, and the first operands of the
// next stage are read behind it during the last quarter, so neither LDS latency nor
// the barrier leaves the matrix cores idle.
// The first step of a tile multiplies into a zero constant instead of clearing
// 256 registers.  The epilogue turns 32-row blocks around in 8 KB of LDS per wave,
// inside the B stage that the tile's last step has finished with and that is filled
// again only by the next step (a barrier after the epilogue keeps it that way).
// A problem may name which 256-row blocks of its output exist (row_bits: frozen row
// blocks of a weight gradient have no tiles) and may continue its contraction over
// the descriptors that follow it (n_seg: layers that share their input give one
// input gradient); the stream treats a new segment like a new tile without epilogue.
//
//   kNT stage: [256 rows][64 contraction] per operand, 16-byte chunks of a row
//              XOR-swizzled; MFMA operands are plain 128-bit LDS reads.
//   kTN stage: [64 contraction][256 rows] per operand (the layout in memory),
//              32-byte units of a row XOR-swizzled; MFMA operands come from the
//              LDS transpose read (4 contraction values of one row per lane).
// A direct-to-LDS load writes lane i's 16 bytes at (wave-uniform base) + 16 i,
// so a swizzle is applied by choosing which global address each lane fetches.
#include "tf_internal.h"

#include <type_traits>
#include <utility>

namespace tf {
namespace {

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kWaves = 4, kThreads = 64 * kWaves;
constexpr int kTileBytes = kBM * kBK * 2;             // 32 KB per operand per stage
// LDS map: three stages of operand B (the "deep" one), two of operand A (the "shallow" one).
// The third stage lets B's loads be issued almost two contraction steps before they are awaited,
// and A's a whole step instead of half a one.  (Which operand is the deep one matters little:
// measured on the two stage shapes, B was better by 1.4 % on one and worse by 0.4 % on the other.)
// The epilogue borrows the deep stage that the tile's last step has just finished with.
constexpr int kDeepStages = 3;
constexpr int kShallowBase = kDeepStages * kTileBytes;            // shallow stages 0, 1 follow the deep ones
constexpr int kEpiBytes = 8192;                                   // per wave, inside the borrowed stage
constexpr int kLdsBytes = (kDeepStages + 2) * kTileBytes;         // 160 KB: all of a compute unit's LDS
static_assert(kWaves * kEpiBytes == kTileBytes, "the four epilogue areas fill one stage");
constexpr int kGroupM = 8;                            // tile rows per L2 locality group
constexpr int kXcds = 8;
constexpr int kXcdRun = 32;                           // consecutive logical tiles kept on one XCD

static_assert(sizeof(GemmBatch) <= 4160, "the batch travels by value in the kernel-argument segment");

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t U2 __attribute__((ext_vector_type(2)));
typedef uint32_t U4 __attribute__((ext_vector_type(4)));
typedef float F4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4* LdsBf16x4Ptr;

#define TF_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N - 1>), in this order
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// two binary32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// Accumulator register -> vector register, at this point of the program.  Left to itself the
// register allocator copies all 256 accumulators of a wave at the head of the epilogue, which
// inside the tile loop is more vector registers than are free.
__device__ __forceinline__ float acc_read(float a) {
    float v;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// Virtual block index -> logical tile.  Hardware hands workgroup b to XCD b % 8, and the
// virtual blocks b, b + gridDim.x, ... of one workgroup keep that XCD (gridDim.x is a
// multiple of 8 whenever a workgroup gets more than one tile).  Runs of kXcdRun consecutive
// logical tiles are kept on one XCD (shared L2), runs go round-robin over the XCDs so that
// all of them work on the same part of the tile list.
// A grid that is not a multiple of 8 (fewer than 8 compute units) keeps the plain order.
__host__ __device__ __forceinline__ int logical_tile(int b, int nb, int grid) {
    const int span = kXcds * kXcdRun;
    const int full = (nb / span) * span;
    if (b >= full || grid % kXcds != 0) return b;
    const int xcd = b % kXcds, idx = b / kXcds;
    return ((idx / kXcdRun) * kXcds + xcd) * kXcdRun + idx % kXcdRun;
}

struct TilePos {
    int pi, m0, n0;            // problem; origin of the 256 x 256 window the tile computes
    // The part of the window that is this tile's to store: rows [r_lo, r_hi), columns [c_lo, c_hi)
    // of the window, (0, 256) x (0, 256) except in a problem's last tile row / column.
    int r_lo, r_hi, c_lo, c_hi;
    __device__ bool whole() const { return r_lo == 0 && r_hi == kBM && c_lo == 0 && c_hi == kBN; }
};

// One dimension of a problem whose extent is not a multiple of the tile edge: where the window
// of its last tile starts and which part of it is stored.  The window is always 256 wide and
// only ever covers operand rows that exist in memory: it is moved back so that it ends with the
// problem (overlapping the tile before it, whose outputs it computes again and does not store);
// a problem narrower than one window may instead run over its end, or start before its
// beginning, by as many rows as the host has said exist there (`before`, `after`).
__device__ __forceinline__ void edge_window(int extent, int tile, int before, int after, int& origin, int& lo, int& hi) {
    origin = tile * kBM; lo = 0; hi = kBM;
    const int missing = origin + kBM - extent;
    if (missing <= 0) return;
    if (after >= missing) { hi = kBM - missing; return; }       // reads past the problem's end, stores what is inside
    origin -= missing;                                          // ends with the problem (origin >= -before)
    lo = missing;
}

// Logical tile -> problem and tile window.  `pi` is where the search starts: a workgroup
// visits its tiles in increasing order, so the problem index never goes back.
__device__ __forceinline__ TilePos locate_tile(const GemmBatch& batch, int lt, int pi) {
    while (pi + 1 < batch.n_problems && lt >= batch.p[pi + 1].tile_start) ++pi;
    const GemmProblem& P = batch.p[pi];
    const int tiles_m = (P.M + kBM - 1) / kBM, tiles_n = (P.N + kBN - 1) / kBN;
    int t = lt - P.tile_start;
    const int per_group = kGroupM * tiles_n;
    const int first_m = (t / per_group) * kGroupM;
    const int gsz = min(tiles_m - first_m, kGroupM);
    t %= per_group;
    int row = first_m + t % gsz;                      // tile row among the rows that exist
    TilePos tp;
    tp.pi = pi;
    if (~P.row_bits != 0) {                           // the row-th set bit is the actual 256-row block (whole tiles only)
        uint64_t b = P.row_bits;
        for (int q = 0; q < row; ++q) b &= b - 1;
        tp.m0 = (__ffsll(static_cast<long long>(b)) - 1) * kBM; tp.r_lo = 0; tp.r_hi = kBM;
    } else {
        edge_window(P.M, row, P.m_slack & 0xffff, P.m_slack >> 16, tp.m0, tp.r_lo, tp.r_hi);
    }
    edge_window(P.N, t / gsz, 0, 0, tp.n0, tp.c_lo, tp.c_hi);
    return tp;
}

// ---------------------------------------------------------------------------------------------
// Stage fill.  Load p of wave w fills KB number (4 p + w) of the 32 KB operand tile.
//   kNT: that KB is tile rows R = 8 (4 p + w) + lane/8, physical chunk lane%8 of each row;
//        logical chunk = physical ^ nt_swizzle(R).
//   kTN: that KB is contraction rows T = 2 (4 p + w) + lane/32, 16-byte slot lane%32 of
//        each; logical 32-byte unit = physical unit ^ (4 ((T / 8) % 4) + T % 4).
// ---------------------------------------------------------------------------------------------
// kNT stage: which physical 16-byte chunk of its 128-byte row holds logical chunk c of tile row R:
// c ^ nt_swizzle(R).  An operand read (ds_read_b128) takes 16 consecutive rows, lane l row l % 16,
// logical chunk l / 16 (+ 4 for the second sub-step).  The LDS serves such a read 16 lanes at a
// time, 8 consecutive lanes together with the 8 lanes 32 further on (counters: with a swizzle that
// only kept 16 consecutive lanes apart, every read took twice its cycles): rows r .. r + 7 of
// chunks q and q ^ 2 must fall into 16 different 16-byte bank groups, and a row's parity already
// selects the half of the banks (row pitch 128 bytes).  Bits 1 and 2 of the row go to bits 0 and 2
// of the swizzle, which the chunk pair does not touch; bit 3 of the row goes to bit 1, which
// also keeps 16 consecutive lanes (one chunk, 16 rows) apart.
__host__ __device__ __forceinline__ constexpr int nt_swizzle(int R) {
    return ((R >> 1) & 1) | (((R >> 3) & 1) << 1) | (((R >> 2) & 1) << 2);
}

struct Side {
    // One operand of a run.  Loads p = 0..3 of a stage fill go through (g, v[p]), loads 4..7
    // through (g2, v[p - 4]).
    const char* g;            // wave-uniform global byte address: tile origin + contraction offset
    const char* g2;
    uint32_t ks;              // byte advance per contraction step of 64 (kTN; a constant for kNT)
    uint32_t v[4];            // per-lane byte offsets; they depend on the row pitch only
};
struct Run {                  // one contraction segment of one tile, as the fill stream sees it
    Side a, b;
    int nk;                   // steps of the segment
};

template <bool kTN>
__device__ __forceinline__ Side make_side(const uint16_t* base, int64_t ld, int origin) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    Side f;
    if (kTN) {
        const int T = 2 * w + (lane >> 5);                     // + 8 p
        const int slot = lane & 31;                            // 16-byte slot of the 512-byte row
        // logical 32-byte unit = physical unit ^ f(T), f(T) = 4 ((T / 8) % 4) + T % 4
        f.g = reinterpret_cast<const char*>(base + origin);
        f.g2 = f.g + 8 * kWaves * ld * 2;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int Tp = T + 2 * kWaves * p;                 // loads p and p + 4 differ by 32 rows: the same f
            const int unit = (slot >> 1) ^ (4 * ((Tp >> 3) & 3) + (Tp & 3));
            f.v[p] = uint32_t((int64_t(Tp) * ld + unit * 16 + (slot & 1) * 8) * 2);
        }
        f.ks = uint32_t(kBK * ld * 2);
    } else {
        const int r = 8 * w + (lane >> 3);                     // + 32 p
        const int pc = lane & 7;
        f.g = reinterpret_cast<const char*>(base + int64_t(origin) * ld);
        f.g2 = f.g + 32 * kWaves * ld * 2;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int R = r + 8 * kWaves * p;
            const int c = pc ^ nt_swizzle(R);                  // the same for p and p + 4
            f.v[p] = uint32_t((int64_t(R) * ld + c * 8) * 2);
        }
        f.ks = 0;
    }
    return f;
}

template <bool kTN>
__device__ __forceinline__ Run make_run(const GemmProblem& P, int m0, int n0) {
    Run f;
    f.a = make_side<kTN>(static_cast<const uint16_t*>(P.A), P.lda, m0);
    f.b = make_side<kTN>(static_cast<const uint16_t*>(P.B), P.ldb, n0);
    f.nk = P.Kc / kBK;
    return f;
}

// One direct-to-LDS load: lane i fetches 16 bytes from gbase + voff and the wave's 1 KB lands
// at LDS byte address lds_wave_base + kLdsOff + 16 i (the LDS address goes through M0).
// Written as inline assembly so that the compiler's wait-count insertion does not treat every
// later LDS read as dependent on it (it would drain the load queue before each transpose read);
// completion is awaited explicitly with wait_direct_loads() before the stage barrier.
// The addition sets SCC, and the compiler is free to place the statement between the two
// halves of one of its own 64-bit scalar additions (s_add_u32 / s_addc_u32) unless it is told:
// a clobbered carry sends the high word of a global address off by one as soon as the addition
// crosses a 4 GiB boundary.  Hence the "scc" clobber; the build scans the generated code for
// inline assembly between a producer and a consumer of SCC and refuses it.  M0 is named for the
// same reason: the compiler keeps values of its own there (LDS-DMA builtins, lane selects).
template <int kLdsOff>
__device__ __forceinline__ void direct_load_16B(const char* gbase, uint32_t voff, uint32_t lds_wave_base) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_wave_base), "v"(voff), "s"(gbase), "n"(kLdsOff)
                 : "memory", "scc", "m0");
}
__device__ __forceinline__ void wait_direct_loads() {
    __builtin_amdgcn_s_waitcnt(0x0f70);     // vmcnt(0), other counters untouched
}

// Load p (0..7) of one operand's stage fill: it fetches KB number 4 p + w of the 32 KB stage.
// lds_stage is the LDS byte address of the stage plus 1 KB times the wave index.  Nothing but
// the load itself: every address is ready in a register.
template <int p>
__device__ __forceinline__ void fill_load(const char* g, const char* g2, const uint32_t (&v)[4], uint32_t lds_stage) {
    direct_load_16B<p * kWaves * 1024>(p < 4 ? g : g2, v[p & 3], lds_stage);
}
template <int p, int end>
__device__ __forceinline__ void fill_side(const Side& f, uint32_t lds_stage) {
    if constexpr (p < end) {
        fill_load<p>(f.g, f.g2, f.v, lds_stage);
        fill_side<p + 1, end>(f, lds_stage);
    }
}

template <class T>
__device__ __forceinline__ T pick(bool c, T a, T b) { return c ? a : b; }
// Byte advance of an operand per contraction step: 64 rows of its pitch, or 64 elements.
template <bool kTN>
__device__ __forceinline__ uint32_t step_bytes(uint32_t ks) { return kTN ? ks : uint32_t(kBK * 2); }

// The fill stream of a workgroup: the contraction segments ("runs") of its tiles, one after the
// other.  `cur` is the run being fetched and `kt` the step inside it whose loads are issued
// next; `nxt` is the run after it, worked out ahead of time so that going from one run to the
// next inside the main loop is a handful of selects and no branch.
struct StreamPos {             // identifies the run held in `nxt`
    int vb;                    // virtual block index of its tile
    int pi;                    // the tile's problem (the first segment's entry)
    int seg, n_seg;            // which contraction segment, segments of the problem
    int m0, n0;                // tile origin
};

template <bool kTN>
__device__ __forceinline__ Run stream_first(StreamPos& c, const GemmBatch& batch, int vb) {
    const TilePos tp = locate_tile(batch, logical_tile(vb, batch.total_tiles, int(gridDim.x)), c.pi);
    c.vb = vb; c.pi = tp.pi; c.m0 = tp.m0; c.n0 = tp.n0;
    c.seg = 0; c.n_seg = batch.p[tp.pi].n_seg;
    return make_run<kTN>(batch.p[c.pi], c.m0, c.n0);
}

// `cur` has just become the run that c identifies (step 0 of it): work out the run after it.
// Past the workgroup's last run the stand-in is that run's last step as a run of its own: it
// is then fetched again, into a stage nobody reads any more, for the two steps by which the
// matrix cores lag behind the stream, which keeps the main loop free of special cases.
template <bool kTN>
__device__ __forceinline__ void stream_prepare(StreamPos& c, const Run& cur, Run& nxt, const GemmBatch& batch) {
    if (c.seg + 1 < c.n_seg) {
        ++c.seg;
        nxt = make_run<kTN>(batch.p[c.pi + c.seg], c.m0, c.n0);
    } else if (c.vb + int(gridDim.x) < batch.total_tiles) {
        nxt = stream_first<kTN>(c, batch, c.vb + int(gridDim.x));
    } else {
        const int64_t last_a = int64_t(cur.nk - 1) * step_bytes<kTN>(cur.a.ks);
        const int64_t last_b = int64_t(cur.nk - 1) * step_bytes<kTN>(cur.b.ks);
        nxt.a.g = cur.a.g + last_a; nxt.a.g2 = cur.a.g2 + last_a;
        nxt.b.g = cur.b.g + last_b; nxt.b.g2 = cur.b.g2 + last_b;
        nxt.a.ks = cur.a.ks; nxt.b.ks = cur.b.ks;
        nxt.nk = 1;
#pragma unroll
        for (int p = 0; p < 4; ++p) { nxt.a.v[p] = cur.a.v[p]; nxt.b.v[p] = cur.b.v[p]; }
    }
}

// Contraction steps of a tile: the sum over its problem's segments.
__device__ __forceinline__ int tile_steps(const GemmBatch& batch, int pi) {
    int n = 0;
    const int n_seg = batch.p[pi].n_seg;
    for (int q = 0; q < n_seg; ++q) n += batch.p[pi + q].Kc / kBK;
    return n;
}

// ---------------------------------------------------------------------------------------------
// MFMA operand fetch.  The MFMA is v_mfma_f32_16x16x32_bf16 (measured from registers with random
// operands, where the chip's power limit decides: 15 % more sustained than the 32x32x16 form, whose
// accumulator traffic per FLOP is twice as large).  Operand lane l holds row (l % 16) of a 16-row
// block and contraction values 8 (l / 16) .. + 7 of the 32 that one instruction contracts; a stage
// holds two such sub-steps u = 0, 1.
// ---------------------------------------------------------------------------------------------
struct FragAddr {
    int a[8], b[8];     // per-lane LDS byte offsets of the 16-row blocks inside a stage of their operand, sub-step 0
};

template <bool kTN>
__device__ __forceinline__ FragAddr make_frag_addr(int wm, int wn) {
    const int lane = threadIdx.x & 63;
    FragAddr fa;
    if (kTN) {
        // LDS transpose read (ds_read_b64_tr_b16): within 16 lanes, result lane i element e comes
        // from source lane 4 e + i / 4, element i % 4.  Lane group G = l / 16 needs contraction rows
        // 8 G .. + 3 (second read: + 4) of the 16 tile rows of its block; as source lane ii it
        // fetches contraction row 8 G + ii / 4, tile rows 4 (ii % 4) .. + 3 (8 bytes).  That row's
        // 32-byte units are XOR-swizzled with 4 G + ii / 4 (make_side), which is different for all
        // 16 rows that one instruction touches: no bank conflicts.
        const int G = lane >> 4, ii = lane & 15;
        const int x = ii >> 2;
        const int laneoff = (8 * G + x) * 512 + 8 * (ii & 3);
#pragma unroll
        for (int i = 0; i < 8; ++i) fa.a[i] = laneoff + (((wm * 8 + i) ^ (4 * G + x)) * 32);
#pragma unroll
        for (int j = 0; j < 8; ++j) fa.b[j] = laneoff + (((wn * 8 + j) ^ (4 * G + x)) * 32);
    } else {
        const int lrow = lane & 15, lq = lane >> 4;
        // chunk (4 u + lq) ^ swz(row): the u-dependent part is XORed in at use
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ra = wm * 128 + i * 16 + lrow;
            fa.a[i] = ra * 128 + ((lq ^ nt_swizzle(ra)) << 4);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int rb = wn * 128 + j * 16 + lrow;
            fa.b[j] = rb * 128 + ((lq ^ nt_swizzle(rb)) << 4);
        }
    }
    return fa;
}

template <bool kTN>
__device__ __forceinline__ bf16x8 load_frag(const char* stage, int addr, int u) {
    if (kTN) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (LdsBf16x4Ptr)TF_LPTR(stage + addr + (32 * u) * 512));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (LdsBf16x4Ptr)TF_LPTR(stage + addr + (32 * u + 4) * 512));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
        // chunk index 4 u + lq, swizzled: 4 u only touches bit 2 of the chunk, lq bits 0..1
        return *reinterpret_cast<const bf16x8*>(stage + (addr ^ (u << 6)));
    }
}

// ---------------------------------------------------------------------------------------------
// Epilogue of one tile, per wave: acc[i][j][e] is C[m][n] with
//   m = row0 + 16 i + lane % 16,  n = col0 + 16 j + 4 (lane / 16) + e.
// A lane's values are scattered over the block, so the wave turns 8 KB pieces around in its
// own LDS area `wlds` (32 rows of 256 bytes) and writes whole 256-byte row segments.
// ---------------------------------------------------------------------------------------------
// kEdge: only rows [r_lo, r_hi) and columns [c_lo, c_hi) of the wave's 128 x 128 block are stored
// (and, when accumulating, read): the tile is the last of its problem in some direction.
template <bool kOutBf16, bool kAccumulate, int kAhead, bool kEdge>
__device__ __forceinline__ void store_block(const f32x4 (&acc)[8][8], char* wlds, void* C, int64_t N,
                                            int row0, int col0, int r_lo = 0, int r_hi = 128, int c_lo = 0, int c_hi = 128) {
    int lane = threadIdx.x & 63;
    // The epilogue sits inside the tile loop.  Its per-lane addresses are loop invariants, and
    // kept in registers across the contraction steps they would crowd out the operands: make
    // the lane number opaque so that they are worked out again for every tile instead.
    asm volatile("" : "+v"(lane));
    const int lrow = lane & 15, lq = lane >> 4;
    const int cb = lane & 15, rsub = lane >> 4;        // 16-byte column block, row inside a group of 4
    if (kOutBf16) {
        // One pass per 32-row block (two 16-row blocks of accumulators): [32 rows][32 chunks of
        // 8 bytes]; the chunk index is XORed with the row so that the rows written by one
        // instruction fall into different banks.
        // Software pipeline: the accumulators of pass i + 1 are read and rounded in between the
        // global stores of pass i, whose rate (the four waves share one path to memory) sets the
        // pace.  The stores are non-temporal: the output is not read again by this kernel, and
        // left in L2 it would push out the operand panels that the other workgroups still fetch.
        uint16_t* Cw = static_cast<uint16_t*>(C) + int64_t(row0) * N + col0 + cb * 8;
        const bool col_ok = !kEdge || (cb * 8 >= c_lo && cb * 8 < c_hi);         // a lane's 8 columns: all or none
        U2 pk[16];                         // one pass, rounded: pk[8 h + j] is chunk 4 j + lq of row 16 h + lrow
        auto round_piece = [&](int ps, int k) {     // two of the sixteen chunks of pass ps
#pragma unroll
            for (int gg = 0; gg < 2; ++gg) {
                const int q = 2 * k + gg, h = q >> 3, j = q & 7;
                const f32x4& a = acc[2 * ps + h][j];
                pk[q] = U2{f32x2_to_bf16x2(acc_read(a[0]), acc_read(a[1])), f32x2_to_bf16x2(acc_read(a[2]), acc_read(a[3]))};
            }
        };
        auto to_lds = [&]() {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int c = 4 * j + lq, r = 16 * h + lrow;
                    *reinterpret_cast<U2*>(wlds + r * 256 + ((c ^ r) << 3)) = pk[8 * h + j];
                }
        };
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; ++k) round_piece(0, k);
        to_lds();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_sched_barrier(0);
            U4 v[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int m = it * 4 + rsub;
                // chunks 2cb and 2cb+1 sit in one aligned 16-byte pair, swapped when m is odd
                v[it] = *reinterpret_cast<const U4*>(wlds + m * 256 + (((2 * cb) ^ (m & ~1)) << 3));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int m = it * 4 + rsub;
                const U4 w = (m & 1) ? U4{v[it].z, v[it].w, v[it].x, v[it].y} : v[it];
                if (!kEdge || (col_ok && i * 32 + m >= r_lo && i * 32 + m < r_hi))
                    __builtin_nontemporal_store(w, reinterpret_cast<U4*>(Cw + int64_t(i * 32 + m) * N));
                if (i < 3) round_piece(i + 1, it);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (i < 3) to_lds();
        }
    } else {
        // fp32: one pass per 32 rows x 64 columns: [32 rows][16 chunks of 16 bytes].  When
        // accumulating, the old values are fetched kAhead passes ahead (two where the registers
        // allow it) so that their HBM latency overlaps the LDS turn-around and the stores.  Old values and results bypass L2
        // retention (non-temporal) for the same reason as above.
        float* Cw = static_cast<float*>(C) + int64_t(row0) * N + col0 + cb * 4;
        auto gaddr = [&](int p, int it) { return Cw + int64_t((p >> 1) * 32 + it * 4 + rsub) * N + (p & 1) * 64; };
        auto mine = [&](int p, int it) {           // is this lane's 4-column piece of pass p, step it, to be stored?
            const int r = (p >> 1) * 32 + it * 4 + rsub, c = (p & 1) * 64 + cb * 4;
            return !kEdge || (r >= r_lo && r < r_hi && c >= c_lo && c < c_hi);
        };
        // (an edge tile fetches each old value right where it is used: no ring of registers)
        constexpr bool kPrefetch = kAccumulate && !kEdge;
        constexpr int kRing = kPrefetch ? kAhead + 1 : 1;
        F4 old[kRing][8];
        auto fetch_old = [&](int p) {
#pragma unroll
            for (int it = 0; it < 8; ++it) old[p % kRing][it] = __builtin_nontemporal_load(reinterpret_cast<const F4*>(gaddr(p, it)));
        };
        if (kPrefetch) {
#pragma unroll
            for (int p = 0; p < kAhead; ++p) fetch_old(p);
        }
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            if (kPrefetch && p + kAhead < 8) fetch_old(p + kAhead);
            const int ps = p >> 1, jh = p & 1;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int c = 4 * jj + lq, r = 16 * h + lrow;
                    const f32x4& a = acc[2 * ps + h][4 * jh + jj];
                    *reinterpret_cast<F4*>(wlds + r * 256 + ((c ^ (r & 15)) << 4)) = F4{a[0], a[1], a[2], a[3]};
                }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int m = it * 4 + rsub;
                F4 v = *reinterpret_cast<const F4*>(wlds + m * 256 + ((cb ^ (m & 15)) << 4));
                if (kPrefetch) v += old[p % kRing][it];
                if (mine(p, it)) {
                    if (kAccumulate && kEdge) v += __builtin_nontemporal_load(reinterpret_cast<const F4*>(gaddr(p, it)));
                    __builtin_nontemporal_store(v, reinterpret_cast<F4*>(gaddr(p, it)));
                }
            }
        }
    }
}

// The same fetch in two halves, for the contraction loop: the LDS address of a fragment (stage
// address, a scalar that changes from step to step, plus the lane's offset) is formed one MFMA
// slot before the read that uses it.  Measured with MFMAs issuing back to back: a vector
// addition followed at once by the LDS read that depends on it holds the wave for 8 cycles
// beyond what the MFMA in flight covers, the read alone for none - with 32 reads per step that
// was a tenth of the step.
template <bool kTN>
__device__ __forceinline__ uint32_t frag_address(uint32_t stage_lds, int addr, int u) {
    uint32_t r;
    const int off = kTN ? addr : (addr ^ (u << 6));
    asm volatile("v_add_u32 %0, %1, %2" : "=v"(r) : "s"(stage_lds), "v"(off));
    return r;
}
template <bool kTN>
__device__ __forceinline__ bf16x8 read_frag(uint32_t a, int u) {
    typedef __attribute__((address_space(3))) const bf16x8* LdsBf16x8Ptr;
    if (kTN) {
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LdsBf16x4Ptr)(uintptr_t)(a + (32 * u) * 512));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LdsBf16x4Ptr)(uintptr_t)(a + (32 * u + 4) * 512));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
        return *(LdsBf16x8Ptr)(uintptr_t)a;
    }
}

// Which operand fragment is read from LDS behind MFMA slot (u, i, jj) of a contraction step.
struct FragRead {
    int op;       // 0 none, 1 an A fragment, 2 a B fragment
    int next;     // 0 this step's stages, 1 the next step's (after the stage barrier)
    int idx;      // 16-row block
    int u;        // sub-step whose operand it is (for a B fragment also the buffer it goes to)
};
__device__ __forceinline__ constexpr FragRead frag_read_at(int u, int i, int jj) {
    // A operand 7 of this very sub-step: its registers were busy until the last row of the
    // sub-step before
    if (i == 0 && jj == 0) return {1, 0, 7, u};
    if (u == 0) {
        // next sub-step, same stage
        if (i >= 1 && jj == 0) return {1, 0, i - 1, 1};
        if (jj == 4) return {2, 0, i, 1};
    } else if (i >= 4) {
        // first sub-step of the next step, after the barrier
        if (i == 4 && !(jj & 1)) return {1, 1, jj >> 1, 0};
        if (i >= 5 && jj == 0) return {1, 1, i - 1, 0};
        if (jj == 1) return {2, 1, 2 * (i - 4), 0};
        if (jj == 5) return {2, 1, 2 * (i - 4) + 1, 0};
    }
    return {0, 0, 0, 0};
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
__global__ __launch_bounds__(kThreads) void gemm_mfma_kernel(GemmBatch batch) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int stride = int(gridDim.x), total = batch.total_tiles;

    // LDS byte address of the dynamic shared array (a 32-bit LDS pointer is its byte offset),
    // plus this wave's 1 KB slot inside every group of 4 KB of a stage fill.
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(uint32_t(reinterpret_cast<uintptr_t>(TF_LPTR(lds))));
    const uint32_t lds_wave_base = lds_base + __builtin_amdgcn_readfirstlane(uint32_t(wave) * 1024u);
    const FragAddr fr = make_frag_addr<kTN>(wm, wn);

    // Fill stream.  The deep operand (B) of step g goes to deep stage g % 3, the shallow operand
    // (A) to shallow stage g % 2.  During step g the loads of the deep operand
    // of step g + 2 are issued in the first quarter (their stage was freed by the barrier of
    // step g - 1) and those of the shallow operand of step g + 2 in the last quarter, right
    // after the barrier that frees its stage.  The barrier of step g needs both operands of step
    // g + 1: everything but the eight youngest loads (the deep operand of step g + 2).  So the
    // deep operand has 1 3/4 steps to arrive and the shallow one a whole step.
    // Both are issued from one position (cur, kt): the deep loads read it directly, then a copy
    // of its shallow side is kept (`lag`) and the position moves on, in the middle of the step,
    // without a branch (the advance pieces below).
    StreamPos pos;
    pos.pi = 0;
    Run cur = stream_first<kTN>(pos, batch, int(blockIdx.x));
    Run nxt;
    stream_prepare<kTN>(pos, cur, nxt, batch);
    int kt = 0;
    bool sw = false;           // the position has just entered a new run
    Side lag;                  // shallow side of the step before the one `cur` stands on

    auto deep = [](Run& r) -> Side& { return r.b; };
    auto shallow = [](Run& r) -> Side& { return r.a; };

    // (cur, kt) -> next step of the stream; in pieces so that each fits beside one MFMA.
    // pick() takes values: a conditional expression over two variables is a choice between
    // their addresses, which would keep them in memory.
    // (the copies are written out so that they stay where they are put: as plain assignments the
    // compiler moves them to the top of the step, into the one slot that has no room)
    auto keep_lag_s = [&]() {
        const Side& sh = shallow(cur);
        asm volatile("s_mov_b64 %0, %1" : "=s"(lag.g) : "s"(sh.g));
        asm volatile("s_mov_b64 %0, %1" : "=s"(lag.g2) : "s"(sh.g2));
    };
    auto keep_lag_v = [&](int h) {
        const Side& sh = shallow(cur);
#pragma unroll
        for (int p = 2 * h; p < 2 * h + 2; ++p) asm volatile("v_mov_b32 %0, %1" : "=v"(lag.v[p]) : "v"(sh.v[p]));
    };
    // Pieces of at most three instructions.  `ahead` holds a pointer one step further on until the
    // next piece decides between it and the new run's.
    const char* ahead;
    auto adv_count = [&]() { ++kt; sw = kt == cur.nk; };
    auto adv_add = [&](const char* g, uint32_t ks) { ahead = g + step_bytes<kTN>(ks); };
    auto adv_sel = [&](const char*& g, const char* n) { g = pick(sw, n, ahead); };
    auto adv_v = [&](Side& c, const Side& n, int p0, int p1) {
#pragma unroll
        for (int p = p0; p < p1; ++p) c.v[p] = pick(sw, n.v[p], c.v[p]);
    };
    auto adv_ks = [&]() {
        if (kTN) {
            cur.a.ks = pick(sw, nxt.a.ks, cur.a.ks);
            cur.b.ks = pick(sw, nxt.b.ks, cur.b.ks);
        }
    };
    auto adv_nk = [&]() {
        cur.nk = pick(sw, nxt.nk, cur.nk);
        kt = pick(sw, 0, kt);
    };
    // piece number n of the position's move (0 .. kAdvancePieces-1)
    constexpr int kAdvancePieces = 15;
    auto advance_piece = [&](int n) {
        switch (n) {
            case 0: adv_count(); break;
            case 1: adv_add(cur.a.g, cur.a.ks); break;
            case 2: adv_sel(cur.a.g, nxt.a.g); break;
            case 3: adv_add(cur.a.g2, cur.a.ks); break;
            case 4: adv_sel(cur.a.g2, nxt.a.g2); break;
            case 5: adv_add(cur.b.g, cur.b.ks); break;
            case 6: adv_sel(cur.b.g, nxt.b.g); break;
            case 7: adv_add(cur.b.g2, cur.b.ks); break;
            case 8: adv_sel(cur.b.g2, nxt.b.g2); break;
            case 9: adv_v(cur.a, nxt.a, 0, 3); break;
            case 10: adv_v(cur.a, nxt.a, 3, 4); adv_v(cur.b, nxt.b, 0, 2); break;
            case 11: adv_v(cur.b, nxt.b, 2, 4); break;
            case 12: adv_ks(); break;
            case 13: adv_nk(); break;
            default: break;
        }
    };
    auto advance = [&]() {
#pragma unroll
        for (int n = 0; n < kAdvancePieces; ++n) advance_piece(n);
    };

    // Steps 0 and 1 in full; the position ends on step 2.
    fill_side<0, 8>(deep(cur), lds_wave_base);
    fill_side<0, 8>(shallow(cur), lds_wave_base + kShallowBase);
    advance();
    if (sw) stream_prepare<kTN>(pos, cur, nxt, batch);
    fill_side<0, 8>(deep(cur), lds_wave_base + kTileBytes);
    fill_side<0, 8>(shallow(cur), lds_wave_base + kShallowBase + kTileBytes);
    advance();
    if (sw) stream_prepare<kTN>(pos, cur, nxt, batch);
    __builtin_amdgcn_s_waitcnt(0x4f70);        // vmcnt(16): step 0 has landed
    __syncthreads();

    // The tile being consumed.
    int cvb = int(blockIdx.x);
    TilePos ct = locate_tile(batch, logical_tile(cvb, total, stride), 0);

    // Stage offsets (bytes from the start of LDS): d0 / s0 hold the step being consumed, d1 / s1
    // the next one, d2 is the deep stage that this step's first quarter fills.
    uint32_t d0 = 0, d1 = kTileBytes, d2 = 2 * kTileBytes;
    uint32_t s0 = kShallowBase, s1 = kShallowBase + kTileBytes;
    auto stage_a = [&](uint32_t, uint32_t sh) { return lds + sh; };     // A is the shallow operand
    auto stage_b = [&](uint32_t d, uint32_t) { return lds + d; };       // B the deep one

    // LDS address of the fragment that the next read fetches (see frag_address): formed behind one
    // MFMA, used behind the next; the one for a step's first read is formed in the last slot of the
    // step before it (here: for the first step).
    uint32_t frag_at = frag_address<kTN>(lds_base + s0, fr.a[7], 0);

    // 8 x 8 accumulator tiles of 16 x 16.  A sub-step (32 of the contraction) is 64 MFMAs, row by
    // row of tiles.  The A operands live in one set of registers: operand i of the next sub-step is
    // read as soon as row i of this one has been issued.  The B operands are needed by every row
    // and are double-buffered.
    f32x4 acc[8][8];
    bf16x8 fa[8], fb[2][8];
#pragma unroll
    for (int i = 0; i < 7; ++i) fa[i] = load_frag<kTN>(stage_a(d0, s0), fr.a[i], 0);
#pragma unroll
    for (int j = 0; j < 8; ++j) fb[0][j] = load_frag<kTN>(stage_b(d0, s0), fr.b[j], 0);

    // Stage offsets of the next step (written out for the same reason as keep_lag).
    uint32_t rot;
    auto rotate_deep = [&](int h) {
        if (h == 0) {
            asm volatile("s_mov_b32 %0, %1" : "=s"(rot) : "s"(d0));
            asm volatile("s_mov_b32 %0, %1" : "=s"(d0) : "s"(d1));
        } else {
            asm volatile("s_mov_b32 %0, %1" : "=s"(d1) : "s"(d2));
            asm volatile("s_mov_b32 %0, %1" : "=s"(d2) : "s"(rot));
        }
    };
    auto rotate_shallow = [&]() {
        uint32_t t;
        asm volatile("s_mov_b32 %0, %1" : "=s"(t) : "s"(s0));
        asm volatile("s_mov_b32 %0, %1" : "=s"(s0) : "s"(s1));
        asm volatile("s_mov_b32 %0, %1" : "=s"(s1) : "s"(t));
    };

    // One contraction step of 64 = two sub-steps u of 64 MFMAs (slot (u, i, jj): row i of tiles,
    // jj-th MFMA of the row).  `first_tag` says whether it opens a tile: then its first sub-step
    // takes a zero constant as addend.  With one wave per SIMD a wave issues one instruction every
    // 4 cycles and an MFMA occupies the matrix pipe for 16: three other instructions fit behind it.
    auto contraction_step = [&](auto first_tag) {
        constexpr bool kFirst = decltype(first_tag)::value;
        // LDS addresses of this step's stages and the next step's: A is the shallow operand, B the deep one
        const uint32_t stage_lds[2][2] = {{lds_base + s0, lds_base + d0}, {lds_base + s1, lds_base + d1}};
        const uint32_t deep_fill = lds_wave_base + d2;
        const uint32_t shallow_fill = lds_wave_base + s0;
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        // Issue order below is pinned with scheduling fences.  The 128 slots are instantiated with
        // their numbers as compile-time constants (no loop to unroll, no index for the compiler to
        // prove constant: every register array is addressed by literals).
        __builtin_amdgcn_sched_barrier(0);
        static_for<128>([&](auto slot_tag) __attribute__((always_inline)) {
            constexpr int slot = decltype(slot_tag)::value;
            constexpr int u = slot >> 6, i = (slot >> 3) & 7, jj = slot & 7;
            if constexpr (u == 1 && i == 4 && jj == 0) {
                // every operand read of this step's stages has been issued: wait for them and
                // for this wave's part of the next step (all loads but the eight issued at the
                // start of this step), then meet the other waves.  After the barrier the next
                // step's stages are complete and this step's may be overwritten.
                __builtin_amdgcn_s_waitcnt(0x0f78);     // vmcnt(8), other counters untouched
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            // boustrophedon over the tiles: consecutive MFMAs always share an operand
            constexpr int j = (i & 1) ? 7 - jj : jj;
            // D rows <- n (B operand rows), D columns <- m: a lane then owns 4 consecutive n
            // of one output row m, i.e. 4 contiguous elements of row-major C.
            if constexpr (kFirst && u == 0)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[u][j], fa[i], zero, 0, 0, 0);
            else
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[u][j], fa[i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);          // the MFMA first, then what rides behind it
            // --- operand reads: this slot's read, from the address formed one slot ago; then
            // the address for the next slot's (the slot after the step's last one is the next
            // step's first, whose stages are this step's next ones) ---
            {
                constexpr FragRead rd = frag_read_at(u, i, jj);
                if constexpr (rd.op == 1) fa[rd.idx] = read_frag<kTN>(frag_at, rd.u);
                if constexpr (rd.op == 2) fb[rd.u][rd.idx] = read_frag<kTN>(frag_at, rd.u);
                constexpr int sl = (slot + 1) % 128;
                constexpr bool wrap = slot == 127;
                constexpr FragRead nx = frag_read_at(sl >> 6, (sl >> 3) & 7, sl & 7);
                if constexpr (nx.op == 1) frag_at = frag_address<kTN>(stage_lds[wrap ? 1 : nx.next][0], fr.a[nx.idx], nx.u);
                if constexpr (nx.op == 2) frag_at = frag_address<kTN>(stage_lds[wrap ? 1 : nx.next][1], fr.b[nx.idx], nx.u);
            }
            // --- stage fills: one load after every fourth MFMA, the rate at which the
            // texture-address unit, which the waves share, takes them ---
            if constexpr (u == 0 && i < 4 && (jj == 2 || jj == 6))        // deep operand of the step after the next
                fill_load<2 * i + (jj >> 2)>(deep(cur).g, deep(cur).g2, deep(cur).v, deep_fill);
            // (the very last slot stays free for the loop's back edge)
            if constexpr (u == 1 && i >= 4 && (jj == 3 || jj == (i == 7 ? 6 : 7)))   // its shallow operand, into the stage just freed
                fill_load<2 * (i - 4) + (jj >> 2)>(lag.g, lag.g2, lag.v, shallow_fill);
            // --- in between, the position moves on: pieces in the slots that hold nothing else ---
            if constexpr (u == 0 && i == 4 && jj == 1) keep_lag_s();
            if constexpr (u == 0 && i == 4 && jj == 2) keep_lag_v(0);
            if constexpr (u == 0 && i == 4 && jj == 3) keep_lag_v(1);
            if constexpr (u == 0 && i >= 5 && jj != 0 && jj != 4) {
                // rows 5, 6, 7: jj = 1, 2, 3, 5, 6, 7 -> pieces 0 .. 17
                constexpr int n = 6 * (i - 5) + (jj < 4 ? jj - 1 : jj - 2);
                if constexpr (n < kAdvancePieces) advance_piece(n);
            }
            if constexpr (u == 1 && i == 0 && jj == 2) rotate_deep(0);     // the step itself works on copies taken at its top
            if constexpr (u == 1 && i == 0 && jj == 3) rotate_deep(1);
            if constexpr (u == 1 && i == 0 && jj == 5) rotate_shallow();
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // Tiles of this workgroup; the inner loop is the hot one.  When the fill position has
    // entered a new run during a step, the run after that one is worked out before the next
    // step: the only decision in the loop, rarely taken, and taken on a counter of its own so
    // that nothing inside a step depends on it.
    int fill_left = cur.nk - kt;                   // steps until the fill position enters a new run
    auto after_step = [&]() {
        if (__builtin_expect(--fill_left == 0, 0)) {
            stream_prepare<kTN>(pos, cur, nxt, batch);
            fill_left = cur.nk;
        }
    };
    for (;;) {
        const int cnk = tile_steps(batch, ct.pi);
        contraction_step(std::true_type{});
        after_step();
        for (int k = 1; k < cnk; ++k) {
            contraction_step(std::false_type{});
            after_step();
        }
        // The deep stage that the last step consumed (d2 after the rotation) is the epilogue's:
        // every wave is past that step's barrier, and its next fill is issued by the next step.
        const GemmProblem& P = batch.p[ct.pi];
        if (__builtin_expect(ct.whole(), 1))
            store_block<kOutBf16, kAccumulate, kTN ? 2 : 1, false>(acc, lds + d2 + wave * kEpiBytes, P.C, P.N,
                                                                   ct.m0 + wm * 128, ct.n0 + wn * 128);
        else
            store_block<kOutBf16, kAccumulate, 1, true>(acc, lds + d2 + wave * kEpiBytes, P.C, P.N,
                                                                  ct.m0 + wm * 128, ct.n0 + wn * 128,
                                                                  ct.r_lo - wm * 128, ct.r_hi - wm * 128,
                                                                  ct.c_lo - wn * 128, ct.c_hi - wn * 128);
        cvb += stride;
        if (cvb >= total) break;
        __syncthreads();          // no wave may fill that stage while another still turns its block around in it
        ct = locate_tile(batch, logical_tile(cvb, total, stride), ct.pi);
    }
    wait_direct_loads();      // nothing of this workgroup may still be in flight towards LDS
}

constexpr int kMaxDevices = 64;

int current_device() {
    int dev = 0;
    return (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) ? dev : -1;
}

int compute_units(int dev) {
    static int cached[kMaxDevices] = {0};
    if (dev < 0) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

template <bool kTN, bool kOutBf16, bool kAccumulate>
hipError_t launch_one(hipStream_t stream, const GemmBatch& batch) {
    auto kern = gemm_mfma_kernel<kTN, kOutBf16, kAccumulate>;
    // the 160 KB of dynamic LDS are allowed once per kernel instantiation and device
    static bool lds_allowed[kMaxDevices] = {false};
    const int dev = current_device();
    if (dev < 0 || !lds_allowed[dev]) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        if (e != hipSuccess) return e;
        if (dev >= 0) lds_allowed[dev] = true;
    }
    hipLaunchKernelGGL(kern, dim3(persistent_grid(batch.total_tiles, compute_units(dev))), dim3(kThreads), kLdsBytes,
                       stream, batch);
    return hipGetLastError();
}

}  // namespace

// One workgroup per compute unit (a workgroup takes all of a unit's LDS and registers).  When a
// workgroup gets more than one tile the grid is a multiple of the XCD count: the tiles b,
// b + grid, ... of a workgroup then keep b % 8, and with it both the XCD and the increasing
// order of logical tiles that the problem search relies on.
int persistent_grid(int total_tiles, int units) {
    if (total_tiles <= units) return total_tiles;
    const int g = units - units % kXcds;
    return g > 0 ? g : units;
}

int gemm_mfma_tile() { return kBM; }

}  // namespace tf

// Test hook (not part of the public header): the order in which a launch of total_tiles tiles on
// `units` compute units walks its tiles.  out[b] = logical tile of virtual block b; returns the
// number of workgroups (workgroup w takes the virtual blocks w, w + grid, ...).
extern "C" int tf_internal_tile_order(int total_tiles, int units, int32_t* out) {
    const int grid = tf::persistent_grid(total_tiles, units);
    for (int b = 0; b < total_tiles; ++b) out[b] = tf::logical_tile(b, total_tiles, grid);
    return grid;
}

namespace tf {

bool mfma_shape_ok(Layout layout, int64_t M, int64_t N, int64_t Kc, int64_t lda, int64_t ldb,
                   int64_t rows_before, int64_t rows_after) {
    // 16-byte direct loads and 16-byte stores: row pitches (C's is N) must keep every row 16-byte
    // aligned, and 256 rows of either operand must lie within the 32-bit per-lane offsets of a stage fill
    constexpr int64_t kMaxPitch = int64_t(1) << 22;
    if (!(M > 0 && N >= kBN && Kc > 0 && Kc % kBK == 0 && N % 8 == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
          lda <= kMaxPitch && ldb <= kMaxPitch))
        return false;
    if (layout == Layout::kTN && M % 8 != 0) return false;           // a window's first column of A stays 16-byte aligned
    return M >= kBM || rows_before + rows_after >= kBM - M;          // a 256-row window must fit into what exists
}

hipError_t launch_gemm_mfma_bf16(hipStream_t stream, GemmBatch& batch, int n_problems,
                                 Layout layout, Dtype out_dtype, bool accumulate) {
    batch.n_problems = n_problems;
    if (n_problems == 0 || batch.total_tiles == 0) return hipSuccess;
    const bool tn = layout == Layout::kTN;
    if (out_dtype == Dtype::BF16)
        return tn ? launch_one<true, true, false>(stream, batch) : launch_one<false, true, false>(stream, batch);
    // fp32 outputs are weight gradients (an input gradient has the inputs' type)
    if (!tn) return hipErrorInvalidValue;
    return accumulate ? launch_one<true, false, true>(stream, batch) : launch_one<true, false, false>(stream, batch);
}

}  // namespace tf
