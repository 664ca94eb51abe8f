// HIP kernels for gfx950 (MI355X, CDNA4, wave64): Y = W.X with W in CER / CSER form
// (Appendix A-C, Algorithms 3 and 4 of the paper) and the constant term for a non-zero most frequent
// value (Appendix A-A1).
//
// Mapping of the method onto the machine
//   * one wavefront owns one output row (times one tile of batch columns);
//   * the wave first turns the row's group pointers into a compact list of its NON-EMPTY groups
//     in LDS: (end offset into colI, value - Omega[0]).  CER derives the value from the group's
//     position in the row, CSER from OmegaI; empty CER padding groups vanish here (ballot +
//     prefix-popcount compaction), so both formats share every later step;
//   * one wave instruction always covers CONSECUTIVE positions of colI (64 of them for batch 1,
//     64/P for a batch tile handled by P lanes per index), so the group structure is wave-uniform:
//     a single cursor in scalar registers walks the row's group boundaries, and only a step whose
//     window contains a boundary does extra work.  Lanes before the boundary add their input to
//     the running sum, every lane multiplies its running sum once by the value of the group that
//     ends, lanes after it start the next sum: one multiplication per (lane, group), never one per
//     element -- the paper's point -- and no lane ever searches a boundary list;
//   * batch = 1: X is staged into LDS once per workgroup and gathered from there; the 64 lane
//     totals are combined with DPP cross-lane adds;
//   * batch > 1: P lanes x V floats cover a tile of batch columns, 64/P indices are gathered per
//     wave instruction from L2 (whole 128-byte rows of X for the default 32-column tile), two
//     batches of gathers are kept in flight; the indices come from one coalesced load per 64
//     positions and a cross-lane read, several batches ahead; workgroups are numbered so that one
//     XCD's L2 sees as few batch tiles of X as possible.  The default batched kernel expands the
//     group values into a per-position array in LDS and multiplies every gathered row by its
//     position's value (no cursor in the stream; a multiply-add costs what an add costs); the
//     cursor variant that sums a group before its one multiplication, and a variant that keeps a
//     narrow tile of X in LDS (reuse of the input), are slower on this machine and opt-in.
// Every load that feeds the streams is unconditional and issued in straight-line code (colI is
// followed by readable padding); positions past a row's end pick up some valid input that lands in
// a running sum multiplied by the list sentinel's weight 0.
// MFMA is not used on this path: it is a gather-accumulate, not a dense contraction.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <numeric>

#include "cer_internal.hpp"

namespace cer {
namespace {

constexpr int kWave = 64;
constexpr uint32_t kNoEnd = 0xFFFFFFFFu;

struct KView {
    const void* colI;
    const uint32_t* omegaPtr;
    const uint32_t* rowPtr;
    const uint2* rowInfo;  // derived: {rowPtr[r], OmegaPtr[rowPtr[r]]}, m + 1 entries
    const void* omegaI;
    const float* omega;
    uint32_t K;
    int32_t omegaI_bits;
    int32_t cser;
    uint32_t m;
    uint32_t n;
    float omega0;
};

// Matrices with rows of unequal length, default batched kernel (kSplit instantiation).  The rows are taken in
// descending order of length (order[i] = the row served i-th), so that the four rows of a workgroup are about
// equally long and the long rows start first.  Rows much longer than the average are served in parts, so that one
// wave does not outlast the whole launch: the row's own work item takes its first `len` positions, every further
// part {row, first position, end position} is a work item of its own (they come first in the grid) whose sums go
// to out[part][batch column] and are added to Y by a second kernel.  nparts == 0: no row is split.
struct SplitArgs {
    const uint32_t* order = nullptr;
    const uint4* parts = nullptr;
    float* out = nullptr;
    uint32_t nparts = 0;
    uint32_t len = 0;          // positions per part
    uint32_t min = 0;          // rows with more positions than this are split
    uint32_t part_blocks = 0;  // workgroups at the front of the grid that serve parts (a multiple of 8)
    const uint4* rows = nullptr;  // host side only: {row, first part, number of parts} per split row
    uint32_t nrows = 0;
};

// OmegaI[g] for an 8-, 16- or 32-bit array, without a branch on the width: the aligned 32-bit
// word that holds the element is loaded and the element is shifted out (the array is padded).
__device__ __forceinline__ uint32_t load_rank(const void* p, int bits, uint32_t g) {
    const uint32_t byte_off = g * ((uint32_t)bits >> 3);
    const uint32_t word = static_cast<const uint32_t*>(p)[byte_off >> 2];
    const uint32_t mask = bits >= 32 ? 0xFFFFFFFFu : ((1u << bits) - 1u);
    return (word >> ((byte_off & 3u) * 8u)) & mask;
}

__device__ __forceinline__ void wave_lds_sync() {
    // LDS operations of one wave are executed in order; only the compiler must not move them.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Sum over the 64 lanes with DPP adds inside each row of 16 lanes, then four lane reads.
__device__ __forceinline__ float wave_sum(float x) {
    auto dpp_add = [](float v, auto ctrl) {
        int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xF, 0xF, false);
        return v + __int_as_float(t);
    };
    x = dpp_add(x, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
    x = dpp_add(x, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
    x = dpp_add(x, std::integral_constant<int, 0x141>{});  // row_half_mirror
    x = dpp_add(x, std::integral_constant<int, 0x140>{});  // row_mirror
    const int xi = __float_as_int(x);
    return (__int_as_float(__builtin_amdgcn_readlane(xi, 0)) + __int_as_float(__builtin_amdgcn_readlane(xi, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(xi, 32)) + __int_as_float(__builtin_amdgcn_readlane(xi, 48)));
}

// ------------------------------------------------------------------------------------------------
// Group list and cursor (shared by both kernels)
// ------------------------------------------------------------------------------------------------

// One lane's share of 64 consecutive raw groups: start, end and rank (Algorithm 3: rank = position
// in the row + 1; Algorithm 4: rank = OmegaI[g]).
struct PtrTile {
    uint32_t s, e, rank;
};

// Loads for raw groups j0 + lane, clamped to the tile so that every lane issues the same
// straight-line loads; lanes past the tile read as an empty group.  OmegaPtr / OmegaI are padded.
__device__ __forceinline__ PtrTile load_ptr_tile(const KView& v, bool cser, uint32_t g0, uint32_t j0, uint32_t tg_end,
                                                 uint32_t lane) {
    const uint32_t g = j0 + lane;
    const uint32_t gc = g < tg_end ? g : (tg_end > j0 ? tg_end - 1u : j0);
    PtrTile p;
    p.s = v.omegaPtr[gc];
    p.e = v.omegaPtr[gc + 1];
    p.rank = cser ? load_rank(v.omegaI, v.omegaI_bits, gc) : gc - g0 + 1u;
    if (g >= tg_end) p.e = p.s;
    return p;
}

// Appends the non-empty groups of one pointer tile to the wave's LDS list (w = that lane's weight).
__device__ __forceinline__ int list_append(const PtrTile& p, float w, uint32_t* ends, float* wts, int count) {
    const bool nonempty = p.e > p.s;
    const uint64_t mask = __ballot(nonempty);
    if (nonempty) {
        const int pos = count + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                               __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        ends[pos] = p.e;
        wts[pos] = w;
    }
    return count + __popcll(mask);
}

// Two sentinels (end = 2^32 - 1, weight 0) close the list: the cursor may sit on the first one.
__device__ __forceinline__ void list_close(uint32_t* ends, float* wts, int count, uint32_t lane) {
    if (lane < 2) {
        ends[count + lane] = kNoEnd;
        wts[count + lane] = 0.f;
    }
}

// List of the non-empty groups among raw groups [tg, tg_end) of the row whose first group is g0.
__device__ __forceinline__ int list_build(const KView& v, bool cser, const float* omega, uint32_t g0, uint32_t tg,
                                          uint32_t tg_end, bool have_first, const PtrTile& first, uint32_t* ends,
                                          float* wts, uint32_t lane) {
    int count = 0;
    for (uint32_t j0 = tg; j0 < tg_end; j0 += kWave) {
        const PtrTile p = (have_first && j0 == tg) ? first : load_ptr_tile(v, cser, g0, j0, tg_end, lane);
        count = list_append(p, omega[p.rank] - v.omega0, ends, wts, count);
    }
    list_close(ends, wts, count, lane);
    return count;
}

// Wave-uniform cursor: current group in scalar registers.  The wave holds 64 consecutive entries of
// its list in two vector registers (lane i = entry chunk + i), so moving on is two lane reads; a row
// with more than 64 non-empty groups reloads the registers from LDS.
struct UCursor {
    uint32_t end;    // colI offset one past the current group (kNoEnd after the last one)
    float w;         // current group's value - Omega[0]
    uint32_t l_end;  // per lane: end of list entry chunk + lane
    float l_w;       // per lane: its value
    int next;        // lane of the entry the cursor takes next, 0 .. 64
    int chunk;       // list index held by lane 0
    int last;        // index of the last list entry (the second sentinel)
};

__device__ __forceinline__ void ucursor_load(UCursor& c, const uint32_t* ends, const float* wts, uint32_t lane) {
    const int i = min(c.chunk + (int)lane, c.last);
    c.l_end = ends[i];
    c.l_w = wts[i];
    c.next = 0;
}

// kFew: the list (sentinels included) fits the 64 lanes, so the registers are never reloaded.
template <bool kFew = false>
__device__ __forceinline__ void ucursor_advance(UCursor& c, const uint32_t* ends, const float* wts, uint32_t lane) {
    if (!kFew && __builtin_expect(c.next == kWave, 0)) {
        c.chunk += kWave;
        ucursor_load(c, ends, wts, lane);
    }
    c.end = __builtin_amdgcn_readlane(c.l_end, c.next);
    c.w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.l_w), c.next));
    ++c.next;
}

__device__ __forceinline__ void ucursor_start(UCursor& c, const uint32_t* ends, const float* wts, int count,
                                              uint32_t lane) {
    c.chunk = 0;
    c.last = count + 1;
    ucursor_load(c, ends, wts, lane);
    ucursor_advance(c, ends, wts, lane);
}

// V batch columns per lane.
template <int V> struct Vec;
template <> struct Vec<1> {
    float a;
    __device__ __forceinline__ void zero() { a = 0.f; }
    __device__ __forceinline__ void add(const Vec& o) { a += o.a; }
    __device__ __forceinline__ void add_if(bool c, const Vec& o) { a += c ? o.a : 0.f; }
    __device__ __forceinline__ void set_if(bool c, const Vec& o) { a = c ? o.a : 0.f; }
    __device__ __forceinline__ void fma(const Vec& r, float w) { a = fmaf(r.a, w, a); }
    __device__ __forceinline__ void fma_if(bool c, const Vec& r, float w) { a = fmaf(c ? r.a : 0.f, w, a); }
    __device__ __forceinline__ void load(const float* p) { a = *p; }
    __device__ __forceinline__ void load_unaligned(const float* p) { a = *p; }
    __device__ __forceinline__ void store(float* p) const { *p = a; }
    __device__ __forceinline__ void xor_add(int off) { a += __shfl_xor(a, off, kWave); }
    __device__ __forceinline__ void add_scaled(const float* t, float s) { a = fmaf(s, t[0], a); }
};
template <> struct Vec<4> {
    float4 a;
    __device__ __forceinline__ void zero() { a = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void add(const Vec& o) { a.x += o.a.x; a.y += o.a.y; a.z += o.a.z; a.w += o.a.w; }
    __device__ __forceinline__ void add_if(bool c, const Vec& o) {
        a.x += c ? o.a.x : 0.f; a.y += c ? o.a.y : 0.f; a.z += c ? o.a.z : 0.f; a.w += c ? o.a.w : 0.f;
    }
    __device__ __forceinline__ void set_if(bool c, const Vec& o) {
        a.x = c ? o.a.x : 0.f; a.y = c ? o.a.y : 0.f; a.z = c ? o.a.z : 0.f; a.w = c ? o.a.w : 0.f;
    }
    __device__ __forceinline__ void fma(const Vec& r, float w) {
        a.x = fmaf(r.a.x, w, a.x); a.y = fmaf(r.a.y, w, a.y); a.z = fmaf(r.a.z, w, a.z); a.w = fmaf(r.a.w, w, a.w);
    }
    __device__ __forceinline__ void fma_if(bool c, const Vec& r, float w) {
        a.x = fmaf(c ? r.a.x : 0.f, w, a.x); a.y = fmaf(c ? r.a.y : 0.f, w, a.y);
        a.z = fmaf(c ? r.a.z : 0.f, w, a.z); a.w = fmaf(c ? r.a.w : 0.f, w, a.w);
    }
    __device__ __forceinline__ void load(const float* p) { a = *reinterpret_cast<const float4*>(p); }
    // the same 16-byte load from an address that is only 4-byte aligned (legal for global memory on this target)
    __device__ __forceinline__ void load_unaligned(const float* p) {
        typedef float F4u __attribute__((ext_vector_type(4), aligned(4)));
        const F4u t = *reinterpret_cast<const F4u*>(p);
        a = make_float4(t.x, t.y, t.z, t.w);
    }
    __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = a; }
    __device__ __forceinline__ void xor_add(int off) {
        a.x += __shfl_xor(a.x, off, kWave); a.y += __shfl_xor(a.y, off, kWave);
        a.z += __shfl_xor(a.z, off, kWave); a.w += __shfl_xor(a.w, off, kWave);
    }
    __device__ __forceinline__ void add_scaled(const float* t, float s) {
        a.x = fmaf(s, t[0], a.x); a.y = fmaf(s, t[1], a.y); a.z = fmaf(s, t[2], a.z); a.w = fmaf(s, t[3], a.w);
    }
};

// One step: the wave instruction covered colI offsets [w0, w0 + WIN); this lane's input x belongs to
// offset w0 + who (who = lane for batch 1, the lane's sub-group for a batch tile).  The current
// group's end is never below w0; the sentinel end (2^32 - 1) is beyond every window.
template <int WIN, int V, bool kFew = false>
__device__ __forceinline__ void cer_step(const Vec<V>& x, uint32_t who, uint32_t w0, UCursor& c, Vec<V>& run,
                                         Vec<V>& acc, const uint32_t* ends, const float* wts, uint32_t lane) {
    if (__builtin_expect(c.end - w0 >= (uint32_t)WIN, 1)) {  // no boundary inside the window
        run.add(x);
        return;
    }
    uint32_t lo = c.end - w0;  // the boundary, as a value of `who`
    run.add_if(who < lo, x);
    acc.fma(run, c.w);  // the one multiplication of this lane for the group that ends here
    ucursor_advance<kFew>(c, ends, wts, lane);
    while (c.end - w0 < (uint32_t)WIN) {  // groups wholly inside the window: at most one element per lane
        const uint32_t hi = c.end - w0;
        acc.fma_if(who >= lo && who < hi, x, c.w);
        lo = hi;
        ucursor_advance<kFew>(c, ends, wts, lane);
    }
    run.set_if(who >= lo, x);
}

// The same step for a batch tile (V > 1 columns per lane).  A window that holds boundaries closes the
// running sum with one multiplication and then lets every lane multiply its own input by its own
// group's value (a fused multiply-add costs what an add costs): per boundary that is one compare and
// one select on a single register instead of selects on all V columns.
template <int WIN, int V>
__device__ __forceinline__ void cer_step_tile(const Vec<V>& x, uint32_t who, uint32_t w0, UCursor& c, Vec<V>& run,
                                              Vec<V>& acc, const uint32_t* ends, const float* wts, uint32_t lane) {
    if (__builtin_expect(c.end - w0 >= (uint32_t)WIN, 1)) {  // no boundary inside the window
        run.add(x);
        return;
    }
    acc.fma(run, c.w);  // what earlier windows gathered for the group that ends here
    run.zero();
    float wl = c.w;
    do {
        const uint32_t lo = c.end - w0;
        ucursor_advance(c, ends, wts, lane);
        wl = who >= lo ? c.w : wl;
    } while (c.end - w0 < (uint32_t)WIN);
    acc.fma(x, wl);
}

// ------------------------------------------------------------------------------------------------
// batch = 1
// ------------------------------------------------------------------------------------------------
//
// Lane l of step s owns the row's (64 s + l)-th index: the index loads are plain coalesced IdxT
// loads (one cache line per wave instruction), all issued before the first is used, and so are the
// LDS gathers of X.  A step without a boundary costs two vector instructions (address shift, add)
// plus the LDS gather; once the stream is in flight the wave's instruction count bounds the kernel.

constexpr int kGemvSteps = 24;  // index loads in flight per lane: one batch covers 64 * 24 positions

// One batch of 24 steps of a row: offsets [b0, b0 + 1536) of colI, whose indices ix[] were requested
// earlier.  The index loads return in order, so step s is gathered and summed while the indices of
// later steps are still on their way from HBM: gathers run eight steps ahead of the sums, and
// scheduling barriers keep the compiler from hoisting every gather (and with it the wait for the
// last index) above the first sum.
template <bool kFew>
__device__ __forceinline__ void gemv_batch(const uint32_t (&ix)[kGemvSteps], const float* xsrc, uint32_t b0, uint32_t te,
                                           uint32_t lane, UCursor& cur, Vec<1>& run, Vec<1>& acc, const uint32_t* ends,
                                           const float* wts) {
    static_assert(kGemvSteps == 24, "steps are spelled out");
    Vec<1> xv[kGemvSteps];
#define CER_GATHER4(S)                                                             \
    xv[S].a = xsrc[ix[S]]; xv[(S) + 1].a = xsrc[ix[(S) + 1]];                      \
    xv[(S) + 2].a = xsrc[ix[(S) + 2]]; xv[(S) + 3].a = xsrc[ix[(S) + 3]];
#define CER_STEP(S) cer_step<kWave, 1, kFew>(xv[S], lane, b0 + (S) * kWave, cur, run, acc, ends, wts, lane)
    // four steps at a time: one boundary test when the next 256 positions hold none
#define CER_STEP4(S)                                                               \
    if (cur.end - (b0 + (S) * kWave) >= 4u * kWave) {                              \
        run.a += (xv[S].a + xv[(S) + 1].a) + (xv[(S) + 2].a + xv[(S) + 3].a);      \
    } else {                                                                       \
        CER_STEP(S); CER_STEP((S) + 1); CER_STEP((S) + 2); CER_STEP((S) + 3);      \
    }
#define CER_PIN __builtin_amdgcn_sched_barrier(0);
    CER_GATHER4(0) CER_GATHER4(4) CER_PIN
    CER_GATHER4(8) CER_PIN CER_STEP4(0) CER_PIN
    CER_GATHER4(12) CER_PIN CER_STEP4(4) CER_PIN
    CER_GATHER4(16) CER_PIN CER_STEP4(8) CER_PIN
    CER_GATHER4(20) CER_PIN
    if (b0 + 12 * kWave < te) {
        CER_STEP4(12)
        if (b0 + 16 * kWave < te) {
            CER_STEP4(16)
            if (b0 + 20 * kWave < te) { CER_STEP4(20) }
        }
    }
#undef CER_PIN
#undef CER_GATHER4
#undef CER_STEP4
#undef CER_STEP
}

// kFew: no row has more than 62 groups (the launcher knows the longest list) and there are at most 64 values, so a
// row's list and its two sentinels fit the cursor's 64 lanes, the cursor never reloads them, and every list is built
// from one pointer tile and a lane shuffle of Omega.
// kOneRow: the launch gives every wave at most one row (matrices of up to 16 rows per compute unit and workgroup
// slot), so the loop over a wave's rows and what it keeps alive fall away.
template <typename IdxT, bool kXinLds, bool kVec4, bool kCser, bool kFew, bool kOneRow>
__global__ __launch_bounds__(1024) void cer_gemv_kernel(KView v, const float* __restrict__ X, float* __restrict__ Y,
                                                        const float* __restrict__ T, uint32_t rows_per_block,
                                                        int omega_in_lds, uint32_t gcap) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NP = kGemvSteps;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t nwaves = blockDim.x >> 6;

    // LDS: [X: n floats, rounded to 4] [Omega: K floats, optional] [ends | wts: nwaves x (gcap + 2)]
    float* xs = reinterpret_cast<float*>(smem);
    const uint32_t x_floats = kXinLds ? ((v.n + 3u) & ~3u) : 0u;
    float* oms = xs + x_floats;
    const uint32_t om_floats = omega_in_lds ? ((v.K + 3u) & ~3u) : 0u;
    uint32_t* list0 = reinterpret_cast<uint32_t*>(oms + om_floats);
    uint32_t* ends = list0 + wave * (gcap + 2);
    float* wts = reinterpret_cast<float*>(list0 + nwaves * (gcap + 2)) + wave * (gcap + 2);
    const float* omega = omega_in_lds ? oms : v.omega;
    const float* xsrc = kXinLds ? xs : X;

    const uint32_t row_begin = blockIdx.x * rows_per_block;
    const uint32_t row_end = min(v.m, row_begin + rows_per_block);
    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    uint32_t r = row_begin + wave;  // wave-uniform: the descriptor loads below are scalar loads

    // (1) descriptor of the wave's first row: {first group, first colI offset} of rows r and r+1
    uint32_t g0 = 0, g1 = 0, rs = 0, re = 0;
    if (r < row_end) {
        const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];
        g0 = d0.x; rs = d0.y; g1 = d1.x; re = d1.y;
    }

    // (2) X and Omega on their way to LDS: eight 16-byte loads per thread are issued here and stay in
    //     flight while the first row's pointers and indices are requested (named registers: an
    //     indexed array would end up in scratch memory)
    typedef float F4 __attribute__((ext_vector_type(4)));
    F4 xr0, xr1, xr2, xr3, xr4, xr5, xr6, xr7;
    const uint32_t n4 = kVec4 ? (v.n >> 2) : 0u;
    const F4* X4 = reinterpret_cast<const F4*>(X);
#define CER_STAGE_IDX(k) ((k) * blockDim.x + threadIdx.x)
#define CER_STAGE_LOAD(k) xr##k = X4[CER_STAGE_IDX(k) < n4 ? CER_STAGE_IDX(k) : n4 - 1u]
    if (kXinLds && kVec4) {  // clamped: every load is issued, none leaves X (the launcher guarantees n4 > 0)
        CER_STAGE_LOAD(0); CER_STAGE_LOAD(1); CER_STAGE_LOAD(2); CER_STAGE_LOAD(3);
        CER_STAGE_LOAD(4); CER_STAGE_LOAD(5); CER_STAGE_LOAD(6); CER_STAGE_LOAD(7);
    }
    const float om_r = v.omega[threadIdx.x < v.K ? threadIdx.x : 0u];
    const float om_l = v.omega[lane < v.K ? lane : 0u];  // Omega[lane]: lets a wave look values up by lane shuffle
    // loads return in issue order: keep the X loads ahead of the index loads, so that staging can finish
    // while the (much longer) index stream is still arriving -- within this wave (scheduling barrier) and
    // within the compute unit, whose memory pipeline is shared by all waves (workgroup barrier: no wave
    // requests indices from HBM before every wave has requested its share of X from L2)
    __builtin_amdgcn_sched_barrier(0);
    if (kXinLds) __syncthreads();
    __builtin_amdgcn_sched_barrier(0);

    // (3) first row: its first 64 group pointers and its first 64 * NP indices, all unconditional
    const PtrTile pt0 = load_ptr_tile(v, kCser, g0, g0, min(g1, g0 + min(gcap, (uint32_t)kWave)), lane);
    uint32_t idx0[NP];  // used by one piece of code only (no merge with re-loaded values, which would make the
                        // compiler widen -- and so wait for -- all of them at the merge point)
    {
        const IdxT* p = colI + rs + lane;
#pragma unroll
        for (int s = 0; s < NP; ++s) idx0[s] = (uint32_t)p[s * kWave];
    }

    __builtin_amdgcn_sched_barrier(0);

    // (4) finish staging
    if (kXinLds) {
        if (kVec4) {
            // all eight values are used here unconditionally, which keeps the compiler from sinking a load
            // into its (conditional) store below the index loads
            asm volatile("" ::"v"(xr0), "v"(xr1), "v"(xr2), "v"(xr3), "v"(xr4), "v"(xr5), "v"(xr6), "v"(xr7));
            F4* xs4 = reinterpret_cast<F4*>(xs);
#define CER_STAGE_STORE(k) if (CER_STAGE_IDX(k) < n4) xs4[CER_STAGE_IDX(k)] = xr##k
            CER_STAGE_STORE(0); CER_STAGE_STORE(1); CER_STAGE_STORE(2); CER_STAGE_STORE(3);
            CER_STAGE_STORE(4); CER_STAGE_STORE(5); CER_STAGE_STORE(6); CER_STAGE_STORE(7);
            for (uint32_t i = 8u * blockDim.x + threadIdx.x; i < n4; i += blockDim.x) xs4[i] = X4[i];
        }
        for (uint32_t i = (n4 << 2) + threadIdx.x; i < v.n; i += blockDim.x) xs[i] = X[i];
    }
#undef CER_STAGE_STORE
#undef CER_STAGE_LOAD
#undef CER_STAGE_IDX
    if (omega_in_lds) {
        if (threadIdx.x < v.K) oms[threadIdx.x] = om_r;
        for (uint32_t i = blockDim.x + threadIdx.x; i < v.K; i += blockDim.x) oms[i] = v.omega[i];
    }
    // With at most 64 values and at most 64 raw groups in the first row, its group list is built
    // here, before the workgroup barrier, from the pointer tile (which arrives ahead of the indices)
    // and a lane shuffle of Omega: the wait for the other waves' share of X hides it.
    int count0 = -1;
    if (kFew || (v.K <= (uint32_t)kWave && g1 - g0 <= min(gcap, (uint32_t)kWave))) {  // kFew: at most 64 values, too
        const float w = __shfl(om_l, (int)(pt0.rank & 63u), kWave) - v.omega0;
        count0 = list_append(pt0, w, ends, wts, 0);
        list_close(ends, wts, count0, lane);
    }
    if (kXinLds || omega_in_lds) __syncthreads();

    // Appendix A-A1: Omega[0] . sum_i X[i].  With X staged in LDS the workgroup sums it there (short per-thread
    // chains, then a tree); otherwise the launcher has computed it into T.
    float t_off = 0.f;
    if (v.omega0 != 0.f) {  // uniform over the grid
        float tsum;
        if (kXinLds) {
            __shared__ float s_part[16];
            float part = 0.f;
            for (uint32_t i = threadIdx.x; i < v.n; i += blockDim.x) part += xs[i];
            part = wave_sum(part);
            if (lane == 0) s_part[wave] = part;
            __syncthreads();
            tsum = 0.f;
            for (uint32_t w = 0; w < nwaves; ++w) tsum += s_part[w];
        } else {
            tsum = T[0];
        }
        t_off = v.omega0 * tsum;
    }

    // The first batch of the first row runs from the prefetched indices when its list is ready
    // (the common case); everything else -- later batches, rows with many groups, later rows --
    // goes through the general loop below, which picks up the cursor and sums where this left off.
    UCursor cur;
    Vec<1> run, acc;
    run.zero();
    acc.zero();
    bool resume = false;
    if (r < row_end && count0 > 0) {
        wave_lds_sync();
        ucursor_start(cur, ends, wts, count0, lane);
        gemv_batch<kFew>(idx0, xsrc, rs, re, lane, cur, run, acc, ends, wts);
        resume = true;
    }

    bool first_row = true;
    for (; r < row_end; r += nwaves) {
        if (!first_row) {
            const uint2 e0 = v.rowInfo[r], e1 = v.rowInfo[r + 1];
            g0 = e0.x; rs = e0.y; g1 = e1.x; re = e1.y;
            acc.zero();
        }
        // a row is one tile unless it has more raw groups than the wave's list holds (never with kFew)
        for (uint32_t tg = g0; tg < g1; tg += gcap) {
            const uint32_t tg_end = kFew ? g1 : min(g1, tg + gcap);
            const uint32_t ts = (kFew || tg == g0) ? rs : uniform(v.omegaPtr[tg]);
            const uint32_t te = (kFew || tg_end == g1) ? re : uniform(v.omegaPtr[tg_end]);
            const bool resumed = first_row && resume;  // single tile, first batch done, list and cursor live
            uint32_t b0 = ts;
            int count;
            if (resumed) {
                count = count0;
                b0 = ts + NP * kWave;
            } else {
                const bool pre = first_row && tg == g0;
                count = ((kFew && kOneRow) || (pre && count0 >= 0))
                            ? count0
                            : list_build(v, kCser, omega, g0, tg, tg_end, pre, pt0, ends, wts, lane);
                wave_lds_sync();
                if (count > 0) ucursor_start(cur, ends, wts, count, lane);
                run.zero();
            }
            if (count > 0) {
                if (b0 < te) {
                    // Two sets of index registers: the next batch is requested before the current one is summed, so
                    // that a wave working alone on a long row (the others of its compute unit are done) does not
                    // wait out the memory latency once per batch.  Past the row's end the current batch is requested
                    // again (in bounds, unused) to keep the loads unconditional.
                    uint32_t ixa[NP], ixb[NP];
#define CER_REQUEST(ix, b)                                                     \
    {                                                                          \
        const IdxT* p_ = colI + (b) + lane;                                    \
        _Pragma("unroll") for (int s = 0; s < NP; ++s) ix[s] = (uint32_t)p_[s * kWave]; \
    }
                    CER_REQUEST(ixa, b0)
                    for (;;) {
                        const uint32_t b1 = b0 + NP * kWave;
                        CER_REQUEST(ixb, b1 < te ? b1 : b0)
                        gemv_batch<kFew>(ixa, xsrc, b0, te, lane, cur, run, acc, ends, wts);
                        if (b1 >= te) break;
                        const uint32_t b2 = b1 + NP * kWave;
                        CER_REQUEST(ixa, b2 < te ? b2 : b1)
                        gemv_batch<kFew>(ixb, xsrc, b1, te, lane, cur, run, acc, ends, wts);
                        if (b2 >= te) break;
                        b0 = b2;
                    }
#undef CER_REQUEST
                }
                acc.fma(run, cur.w);
            }
            wave_lds_sync();  // the list is rebuilt by the next tile / row
            if (kFew) break;  // one tile per row
        }
        const float y = wave_sum(acc.a);
        if (lane == 0) Y[r] = y + t_off;
        if (kOneRow) break;
        first_row = false;
    }
}

// ------------------------------------------------------------------------------------------------
// batch > 1
// ------------------------------------------------------------------------------------------------

constexpr int kGemmGroupTile = 256;  // raw groups turned into one LDS list at a time

// Index registers of the batched kernel.  One register holds the indices of 64 consecutive colI
// positions (one coalesced load per wave); a wave instruction of the gather needs only S = 64/P of
// them, which every lane fetches from the register by a cross-lane read.  A batch of U windows
// covers PB = U.S positions = KQ registers, and D batches of indices are kept in flight.
template <int P>
struct GemmIdx {
    static constexpr int S = kWave / P, U = 8, PB = U * S;
    static constexpr int KQ = PB >= kWave ? PB / kWave : 1;
    static constexpr int D = KQ == 1 ? 8 : (KQ <= 4 ? 4 : 2);
};

// The stream of one tile of groups, colI offsets [ts, te): while one batch of U windows is summed,
// the gathers of the next batch and the index loads D batches ahead are under way.  With kPre the
// index registers of the first D batches were requested by the caller.
template <typename IdxT, int V, int P, bool kPre>
__device__ __forceinline__ void gemm_tile(const IdxT* colI, const float* xgather, uint32_t L, uint32_t ts, uint32_t te,
                                          uint32_t sub, uint32_t lane, uint32_t (&iq)[GemmIdx<P>::D][GemmIdx<P>::KQ],
                                          UCursor& cur, Vec<V>& run, Vec<V>& acc, const uint32_t* ends, const float* wts) {
    using G = GemmIdx<P>;
    constexpr int S = G::S, U = G::U, KQ = G::KQ, D = G::D;
    constexpr uint32_t PB = G::PB;
    Vec<V> xa[U], xb[U];
#define CER_LOADQ(d, b) \
    _Pragma("unroll") for (int q = 0; q < KQ; ++q) iq[d][q] = (uint32_t)colI[(b) + q * kWave + lane];
#define CER_GATHER(xv, d)                                                                             \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                   \
        const uint32_t reg_ = iq[d][(u * S) / kWave];                                                 \
        const uint32_t idx_ = S == kWave ? reg_ : (uint32_t)__shfl((int)reg_, (int)((u * S) % kWave + sub), kWave); \
        xv[u].load(xgather + (size_t)idx_ * L);                                                       \
    }
#define CER_CONSUME(xv, b) \
    _Pragma("unroll") for (int u = 0; u < U; ++u) cer_step_tile<S, V>(xv[u], sub, (b) + u * S, cur, run, acc, ends, wts, lane);
#define CER_STEP(xcur, xnext, dn, dl, k)   \
    CER_GATHER(xnext, dn)                  \
    CER_LOADQ(dl, base + ((k) + D) * PB)   \
    CER_CONSUME(xcur, base + (k) * PB)
    if (!kPre) {
        _Pragma("unroll") for (int d = 0; d < D; ++d) { CER_LOADQ(d, ts + d * PB) }
    }
    CER_GATHER(xa, 0)
    for (uint32_t base = ts; base < te; base += D * PB) {
        CER_STEP(xa, xb, 1 % D, 0, 0)
        if (D > 2 && base + PB >= te) break;
        CER_STEP(xb, xa, 2 % D, 1 % D, 1)
        if (D > 2) {
            if (base + 2 * PB >= te) break;
            CER_STEP(xa, xb, 3 % D, 2 % D, 2)
            if (base + 3 * PB >= te) break;
            CER_STEP(xb, xa, 4 % D, 3 % D, 3)
        }
        if (D > 4) {
            if (base + 4 * PB >= te) break;
            CER_STEP(xa, xb, 5 % D, 4 % D, 4)
            if (base + 5 * PB >= te) break;
            CER_STEP(xb, xa, 6 % D, 5 % D, 5)
            if (base + 6 * PB >= te) break;
            CER_STEP(xa, xb, 7 % D, 6 % D, 6)
            if (base + 7 * PB >= te) break;
            CER_STEP(xb, xa, 0, 7 % D, 7)
        }
    }
#undef CER_LOADQ
#undef CER_GATHER
#undef CER_CONSUME
#undef CER_STEP
}

// V floats per lane, P lanes per index: one wave instruction gathers 64/P rows of X, each
// V.P floats wide.  Workgroup = 4 waves = 4 consecutive rows of one batch tile.
template <typename IdxT, int V, int P>
__global__ __launch_bounds__(256) void cer_gemm_kernel(KView v, const float* __restrict__ X, float* __restrict__ Y,
                                                       const float* __restrict__ T, uint32_t L, uint32_t ntiles,
                                                       uint32_t rowblocks, uint32_t items_per_xcd) {
    constexpr int TW = V * P;  // batch columns per tile; a wave instruction covers 64 / P colI positions
    __shared__ uint32_t s_ends[4][kGemmGroupTile + 2];
    __shared__ float s_wts[4][kGemmGroupTile + 2];

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give XCD x the x-th
    // eighth of the (tile-major) work list, so that an XCD walks through few batch tiles of X.
    const uint32_t xcd = blockIdx.x & 7u, q = blockIdx.x >> 3;
    const uint32_t nitems = ntiles * rowblocks;
    const uint32_t item = xcd * items_per_xcd + q;
    if (q >= items_per_xcd || item >= nitems) return;
    const uint32_t tile = item / rowblocks;
    const uint32_t r = (item - tile * rowblocks) * 4u + wave;
    if (r >= v.m) return;

    const uint32_t sub = lane / P;
    const uint32_t col0 = tile * TW + (lane % P) * V;
    const bool active = col0 < L;  // V = 4 requires L % 4 == 0, so a lane is all in or all out
    const float* xgather = X + (active ? col0 : 0u);  // lanes beyond the batch read column 0 and store nothing
    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    uint32_t* ends = s_ends[wave];
    float* wts = s_wts[wave];

    const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];  // scalar loads: r is wave-uniform
    const uint32_t g0 = d0.x, rs = d0.y, g1 = d1.x, re = d1.y;
    // Everything the first tile needs is requested at once -- 64 group pointers, Omega by lane, the
    // indices of the first batches -- so that their latencies overlap instead of adding up.
    const bool cser = v.cser != 0;
    const uint32_t tg_end0 = min(g1, g0 + (uint32_t)kGemmGroupTile);
    const PtrTile pt0 = load_ptr_tile(v, cser, g0, g0, min(tg_end0, g0 + (uint32_t)kWave), lane);
    const float om_l = v.omega[lane < v.K ? lane : 0u];
    uint32_t iq[GemmIdx<P>::D][GemmIdx<P>::KQ];
#pragma unroll
    for (int d = 0; d < GemmIdx<P>::D; ++d)
#pragma unroll
        for (int q = 0; q < GemmIdx<P>::KQ; ++q) iq[d][q] = (uint32_t)colI[rs + d * GemmIdx<P>::PB + q * kWave + lane];

    Vec<V> acc, run;
    acc.zero();
    UCursor cur;
    if (g1 > g0) {
        const uint32_t te = (tg_end0 == g1) ? re : uniform(v.omegaPtr[tg_end0]);
        int count;
        if (v.K <= (uint32_t)kWave && tg_end0 - g0 <= (uint32_t)kWave) {  // values looked up by lane shuffle
            count = list_append(pt0, __shfl(om_l, (int)(pt0.rank & 63u), kWave) - v.omega0, ends, wts, 0);
            list_close(ends, wts, count, lane);
        } else {
            count = list_build(v, cser, v.omega, g0, g0, tg_end0, true, pt0, ends, wts, lane);
        }
        wave_lds_sync();
        if (count > 0) {
            ucursor_start(cur, ends, wts, count, lane);
            run.zero();
            gemm_tile<IdxT, V, P, true>(colI, xgather, L, rs, te, sub, lane, iq, cur, run, acc, ends, wts);
            acc.fma(run, cur.w);
        }
        wave_lds_sync();
    }
    // rows with more raw groups than one list holds: further tiles
    for (uint32_t tg = g0 + kGemmGroupTile; tg < g1; tg += kGemmGroupTile) {
        const uint32_t tg_end = min(g1, tg + kGemmGroupTile);
        const uint32_t ts = uniform(v.omegaPtr[tg]);
        const uint32_t te = (tg_end == g1) ? re : uniform(v.omegaPtr[tg_end]);
        const int count = list_build(v, cser, v.omega, g0, tg, tg_end, false, pt0, ends, wts, lane);
        wave_lds_sync();
        if (count > 0) {
            ucursor_start(cur, ends, wts, count, lane);
            run.zero();
            gemm_tile<IdxT, V, P, false>(colI, xgather, L, ts, te, sub, lane, iq, cur, run, acc, ends, wts);
            acc.fma(run, cur.w);
        }
        wave_lds_sync();
    }
#pragma unroll
    for (int off = P; off < kWave; off <<= 1) acc.xor_add(off);
    if (sub == 0 && active) {
        if (v.omega0 != 0.f) acc.add_scaled(T + col0, v.omega0);
        acc.store(Y + (size_t)r * L + col0);
    }
}

// ------------------------------------------------------------------------------------------------
// batch > 1, the default kernel: group values expanded per position
// ------------------------------------------------------------------------------------------------
//
// Finding group ends inside the index stream costs instructions in every window, and in rows made of
// short groups nearly every window holds boundaries.  Here the group structure is expanded once per
// chunk of 2048 colI positions into a per-position value array in LDS (long groups are written by the
// whole wave, short ones by one lane each); the stream is then a plain multiply-add of each gathered
// input row by its position's value, with no data-dependent control flow.  Summing a group before its
// one multiplication saves nothing on this machine -- a fused multiply-add costs what an add costs --
// so this kernel beat the cursor kernel above on every measured workload, not only on short groups.

// Writes the columns colx .. colx + 3 of a row that are not below `first` (the lane's nominal first column).
__device__ __forceinline__ void ragged_store(const Vec<4>& acc, float* yrow, const float* T, float omega0, uint32_t colx,
                                             uint32_t first) {
    const float o[4] = {acc.a.x, acc.a.y, acc.a.z, acc.a.w};
#pragma unroll
    for (uint32_t e = 0; e < 4; ++e) {
        const uint32_t c = colx + e;
        if (c >= first) yrow[c] = omega0 != 0.f ? fmaf(omega0, T[c], o[e]) : o[e];
    }
}
__device__ __forceinline__ void ragged_store(const Vec<1>&, float*, const float*, float, uint32_t, uint32_t) {}

// colI positions whose values one expansion holds: 2048 (8 KiB per wave), or 512 for matrices of short rows, whose
// waves are bound by their start-up chain and gain from six instead of four workgroups per compute unit
constexpr int kExpChunkLong = 2048, kExpChunkShort = 512;
constexpr uint32_t kExpLong = 16;  // groups longer than this are written by the whole wave

// kRagged (V = 4 only): the batch width is not a multiple of 4 or X / Y are only 4-byte aligned.  The gathers are
// 16-byte loads from 4-byte aligned addresses; the lanes of the last, partial column group take the row's last four
// columns instead (all loads stay inside the row) and write only the columns no other lane owns; Y is written
// element by element.
template <typename IdxT, int V, int P, bool kRagged, int kExpChunk = kExpChunkLong, bool kSplit = false>
__global__ __launch_bounds__(256) void cer_gemm_expand_kernel(KView v, const float* __restrict__ X, float* __restrict__ Y,
                                                              const float* __restrict__ T, uint32_t L, uint32_t ntiles,
                                                              uint32_t rowblocks, uint32_t items_per_xcd, SplitArgs sp) {
    using G = GemmIdx<P>;
    constexpr int S = G::S, U = G::U, KQ = G::KQ, D = G::D;
    constexpr uint32_t PB = G::PB;
    constexpr uint32_t PAD = D * PB;  // the last loop body of a chunk reads (zero) values this far past its end
    constexpr int TW = V * P;
    __shared__ float s_val[4][kExpChunk + PAD];

    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    uint32_t tile, r;
    uint32_t part = 0, part_begin = 0, part_end = 0;
    const bool is_part = kSplit && blockIdx.x < sp.part_blocks;  // a further part of a long row
    if (is_part) {
        const uint32_t e = blockIdx.x * 4u + wave;  // tile-major over (tile, part)
        if (e >= ntiles * sp.nparts) return;
        tile = e / sp.nparts;
        part = e - tile * sp.nparts;
        const uint4 d = sp.parts[part];
        r = uniform(d.x);
        part_begin = uniform(d.y);
        part_end = uniform(d.z);
    } else {
        const uint32_t b = kSplit ? blockIdx.x - sp.part_blocks : blockIdx.x;  // part_blocks is a multiple of 8
        const uint32_t xcd = b & 7u, q = b >> 3;
        const uint32_t nitems = ntiles * rowblocks;
        const uint32_t item = xcd * items_per_xcd + q;
        if (q >= items_per_xcd || item >= nitems) return;
        tile = item / rowblocks;
        const uint32_t rb = item - tile * rowblocks;
        if (kSplit) {
            // Rows by descending length.  S XCDs share a batch tile, each walking a contiguous range of rb: deal the
            // length ranks round-robin to those ranges (range j takes ranks j, j + S, ...), so that every XCD gets
            // rows of every length and meets them longest first.
            const uint32_t S = ntiles >= 8u ? 1u : 8u / ntiles;
            const uint32_t q0 = rowblocks / S, rem = rowblocks - q0 * S;
            uint32_t rank_block = rb;
            if (S > 1u && q0 > 0u) {
                uint32_t i, j;
                if (rb < rem * (q0 + 1u)) {
                    j = rb / (q0 + 1u);
                    i = rb - j * (q0 + 1u);
                } else {
                    const uint32_t rb2 = rb - rem * (q0 + 1u);
                    j = rb2 / q0;
                    i = rb2 - j * q0;
                    j += rem;
                }
                rank_block = i * S + j;
            }
            const uint32_t rank = rank_block * 4u + wave;
            if (rank >= v.m) return;
            r = uniform(sp.order[rank]);
        } else {
            r = rb * 4u + wave;
            if (r >= v.m) return;
        }
    }

    const uint32_t sub = lane / P;
    const uint32_t col0 = tile * TW + (lane % P) * V;
    const bool active = col0 < L;
    static_assert(!kRagged || V == 4, "ragged batches are gathered four columns at a time");
    const uint32_t colx = kRagged ? min(col0, L - 4u) : col0;  // ragged: L >= 4 (the launcher sees to it)
    const float* xgather = X + (active ? colx : 0u);
    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    float* val = s_val[wave];

    const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];
    const uint32_t g0 = d0.x, g1 = d1.x;
    uint32_t rs = d0.y, re = d1.y;
    if (kSplit) {  // a part's own positions; the first part of a split row
        if (is_part) {
            rs = part_begin;
            re = part_end;
        } else if (re - rs > sp.min) {
            re = rs + sp.len;
        }
    }
    const bool cser = v.cser != 0;
    const float om_l = v.omega[lane < v.K ? lane : 0u];
    const bool omega_by_lane = v.K <= (uint32_t)kWave;

    Vec<V> acc;
    acc.zero();
    uint32_t gcur = g0;  // first raw group that may reach into the current chunk (groups that end before it cost
                         // a part nothing but their pointer tiles)
    for (uint32_t c0 = rs; c0 < re; c0 += kExpChunk) {
        const uint32_t c1 = min(re, c0 + (uint32_t)kExpChunk);
        // request order = arrival order: the chunk's first 64 group pointers, then its indices, then (below) the
        // first gathers; the expansion then waits for the pointers only and runs under the gathers' L2 latency
        const PtrTile p_first = load_ptr_tile(v, cser, g0, gcur, g1, lane);
        const uint32_t g_first = gcur;
        uint32_t iq[D][KQ];
#pragma unroll
        for (int d = 0; d < D; ++d)
#pragma unroll
            for (int qq = 0; qq < KQ; ++qq) iq[d][qq] = (uint32_t)colI[c0 + d * PB + qq * kWave + lane];

        Vec<V> xa[U], xb[U];
#define CER_LOADQ(d, b) \
    _Pragma("unroll") for (int qq = 0; qq < KQ; ++qq) iq[d][qq] = (uint32_t)colI[(b) + qq * kWave + lane];
#define CER_GATHER(xv, d)                                                                             \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                   \
        const uint32_t reg_ = iq[d][(u * S) / kWave];                                                 \
        const uint32_t idx_ = S == kWave ? reg_ : (uint32_t)__shfl((int)reg_, (int)((u * S) % kWave + sub), kWave); \
        if (kRagged) xv[u].load_unaligned(xgather + (size_t)idx_ * L); else xv[u].load(xgather + (size_t)idx_ * L); \
    }
#define CER_CONSUME(xv, b) \
    _Pragma("unroll") for (int u = 0; u < U; ++u) acc.fma(xv[u], val[(b) - c0 + u * S + sub]);
#define CER_STEP(xcur, xnext, dn, dl, k)   \
    CER_GATHER(xnext, dn)                  \
    CER_LOADQ(dl, base + ((k) + D) * PB)   \
    CER_CONSUME(xcur, base + (k) * PB)
        CER_GATHER(xa, 0)

        // ---- expansion: value of every position of [c0, c1); zeros behind it
        for (uint32_t i = c1 - c0 + lane; i < min(c1 - c0 + PAD, (uint32_t)kExpChunk + PAD); i += kWave) val[i] = 0.f;
        for (uint32_t gt = gcur; gt < g1; gt += kWave) {
            const PtrTile p = gt == g_first ? p_first : load_ptr_tile(v, cser, g0, gt, g1, lane);
            const float w = (omega_by_lane ? __shfl(om_l, (int)(p.rank & 63u), kWave) : v.omega[p.rank < v.K ? p.rank : 0u]) - v.omega0;
            const uint32_t s = max(p.s, c0), e = min(p.e, c1);
            const uint32_t len = e > s ? e - s : 0u;
            uint64_t longs = __ballot(len > kExpLong);
            while (longs) {
                const int b = __builtin_ctzll(longs);
                longs &= longs - 1;
                const uint32_t s_b = __builtin_amdgcn_readlane(s, b), e_b = __builtin_amdgcn_readlane(e, b);
                const float w_b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), b));
                for (uint32_t pos = s_b + lane; pos < e_b; pos += kWave) val[pos - c0] = w_b;
            }
            if (len <= kExpLong) {
#pragma unroll
                for (uint32_t k = 0; k < kExpLong; ++k)
                    if (k < len) val[s - c0 + k] = w;
            }
            // groups of this tile that end inside the chunk are done with
            const uint32_t done = (uint32_t)__popcll(__ballot(gt + lane < g1 && p.e <= c1));
            gcur = gt + done;
            if (done < (uint32_t)kWave) break;  // the next group reaches beyond the chunk (or the row is finished)
        }
        wave_lds_sync();

        // ---- stream of the chunk: multiply every gathered row by its position's value, add
        for (uint32_t base = c0; base < c1; base += D * PB) {
            CER_STEP(xa, xb, 1 % D, 0, 0)
            if (D > 2 && base + PB >= c1) break;
            CER_STEP(xb, xa, 2 % D, 1 % D, 1)
            if (D > 2) {
                if (base + 2 * PB >= c1) break;
                CER_STEP(xa, xb, 3 % D, 2 % D, 2)
                if (base + 3 * PB >= c1) break;
                CER_STEP(xb, xa, 4 % D, 3 % D, 3)
            }
            if (D > 4) {
                if (base + 4 * PB >= c1) break;
                CER_STEP(xa, xb, 5 % D, 4 % D, 4)
                if (base + 5 * PB >= c1) break;
                CER_STEP(xb, xa, 6 % D, 5 % D, 5)
                if (base + 6 * PB >= c1) break;
                CER_STEP(xa, xb, 7 % D, 6 % D, 6)
                if (base + 7 * PB >= c1) break;
                CER_STEP(xb, xa, 0, 7 % D, 7)
            }
        }
#undef CER_LOADQ
#undef CER_GATHER
#undef CER_CONSUME
#undef CER_STEP
        wave_lds_sync();  // the next chunk overwrites the values
    }
#pragma unroll
    for (int off = P; off < kWave; off <<= 1) acc.xor_add(off);
    if (sub == 0 && active) {
        if (kSplit && is_part) {  // partial sums of a further part: no constant term
            if (kRagged) ragged_store(acc, sp.out + (size_t)part * L, T, 0.f, colx, col0);
            else acc.store(sp.out + (size_t)part * L + col0);
        } else if (kRagged) {
            ragged_store(acc, Y + (size_t)r * L, T, v.omega0, colx, col0);
        } else {
            if (v.omega0 != 0.f) acc.add_scaled(T + col0, v.omega0);
            acc.store(Y + (size_t)r * L + col0);
        }
    }
}

// Y[row] += the sums of the row's further parts, in the order of the parts (deterministic).  One workgroup per
// split row; rows[i] = {row, first part, number of parts}.
__global__ __launch_bounds__(256) void split_add_kernel(const uint4* __restrict__ rows, const float* __restrict__ part_out,
                                                        float* __restrict__ Y, uint32_t L) {
    const uint4 d = rows[blockIdx.x];
    for (uint32_t c = threadIdx.x; c < L; c += blockDim.x) {
        float s = Y[(size_t)d.x * L + c];
        for (uint32_t p = 0; p < d.z; ++p) s += part_out[(size_t)(d.y + p) * L + c];
        Y[(size_t)d.x * L + c] = s;
    }
}

// ------------------------------------------------------------------------------------------------
// batch = 1, rows made of many short groups
// ------------------------------------------------------------------------------------------------
//
// With hundreds of values per row (8-bit codebooks) a group holds a handful of elements and the cursor of
// the kernel above crosses several group ends in every window of 64 positions.  This kernel expands the group
// structure instead, as the default batched kernel does: per chunk of kGemvExpChunk colI positions the value of
// every position goes to an array in LDS (long groups written by the whole wave, short ones by one lane each) and
// the stream is acc += X[colI[p]] . val[p], lane = position, X staged in LDS.  One wave per row; the index loads
// of a chunk are issued before its expansion starts and run into the next row or the padding behind colI.

constexpr uint32_t kGemvExpShort = 32;  // groups up to this length are written by one lane each, longer ones by the whole wave

// kGemvExpChunk = positions per expansion: 2048 (32 index registers per lane, 8 KiB of values per wave), or 512 for
// matrices of short rows, whose waves then leave room in LDS for several workgroups per compute unit
template <typename IdxT, bool kCser, uint32_t kGemvExpChunk>
__global__ __launch_bounds__(1024) void cer_gemv_expand_kernel(KView v, const float* __restrict__ X, float* __restrict__ Y,
                                                               uint32_t rows_per_block, int omega_in_lds) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr uint32_t NW = kGemvExpChunk / kWave;  // windows per chunk
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t nwaves = blockDim.x >> 6;

    // LDS: [X: n floats, rounded to 4][Omega: K floats, optional][values: nwaves x (chunk + 64)]
    float* xs = reinterpret_cast<float*>(smem);
    const uint32_t x_floats = (v.n + 3u) & ~3u;
    float* oms = xs + x_floats;
    const uint32_t om_floats = omega_in_lds ? ((v.K + 3u) & ~3u) : 0u;
    float* val = oms + om_floats + wave * (kGemvExpChunk + kWave);
    const float* omega = omega_in_lds ? oms : v.omega;

    if ((reinterpret_cast<uintptr_t>(X) & 15u) == 0) {
        const float4* X4 = reinterpret_cast<const float4*>(X);
        float4* xs4 = reinterpret_cast<float4*>(xs);
        const uint32_t n4 = v.n >> 2;
        for (uint32_t i = threadIdx.x; i < n4; i += blockDim.x) xs4[i] = X4[i];
        for (uint32_t i = (n4 << 2) + threadIdx.x; i < v.n; i += blockDim.x) xs[i] = X[i];
    } else {
        for (uint32_t i = threadIdx.x; i < v.n; i += blockDim.x) xs[i] = X[i];
    }
    if (omega_in_lds)
        for (uint32_t i = threadIdx.x; i < v.K; i += blockDim.x) oms[i] = v.omega[i];
    __syncthreads();

    // Appendix A-A1: Omega[0] . sum_i X[i], summed from the staged copy
    float t_off = 0.f;
    if (v.omega0 != 0.f) {  // uniform over the grid
        __shared__ float s_part[16];
        float part = 0.f;
        for (uint32_t i = threadIdx.x; i < v.n; i += blockDim.x) part += xs[i];
        part = wave_sum(part);
        if (lane == 0) s_part[wave] = part;
        __syncthreads();
        float tsum = 0.f;
        for (uint32_t w = 0; w < nwaves; ++w) tsum += s_part[w];
        t_off = v.omega0 * tsum;
    }

    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    const bool cser = kCser;
    const uint32_t row_begin = blockIdx.x * rows_per_block;
    const uint32_t row_end = min(v.m, row_begin + rows_per_block);
    for (uint32_t r = row_begin + wave; r < row_end; r += nwaves) {  // wave-uniform
        const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];
        const uint32_t g0 = d0.x, rs = d0.y, g1 = d1.x, re = d1.y;
        float acc = 0.f;
        uint32_t gcur = g0;  // first raw group that may reach into the current chunk
        // the pointers of the row's first 256 raw groups are requested together (tiles past the row's last group read
        // the padding behind the pointer arrays and come back empty)
        constexpr int kPre = 4;
        PtrTile pre[kPre];
#pragma unroll
        for (int t = 0; t < kPre; ++t) pre[t] = load_ptr_tile(v, cser, g0, min(g0 + (uint32_t)t * kWave, g1), g1, lane);
        for (uint32_t c0 = rs; c0 < re; c0 += kGemvExpChunk) {
            const uint32_t c1 = min(re, c0 + kGemvExpChunk);
            const uint32_t nwin = (c1 - c0 + kWave - 1u) / kWave;
            uint32_t ix[NW];
#pragma unroll
            for (uint32_t w = 0; w < NW; ++w) ix[w] = (uint32_t)colI[c0 + w * kWave + lane];

            // values of the positions [c0, c1), zeros up to the end of the last window
            if (c1 - c0 + lane < nwin * kWave) val[c1 - c0 + lane] = 0.f;
            // one tile of 64 raw groups starting at gt; false: the next group reaches beyond the chunk or the row is done
            auto expand_tile = [&](const PtrTile& p, uint32_t gt) {
                const float w = omega[p.rank < v.K ? p.rank : 0u] - v.omega0;
                const uint32_t s = max(p.s, c0), e = min(p.e, c1);
                const uint32_t len = e > s ? e - s : 0u;
                uint64_t longs = __ballot(len > kGemvExpShort);
                while (longs) {
                    const int b = __builtin_ctzll(longs);
                    longs &= longs - 1;
                    const uint32_t s_b = __builtin_amdgcn_readlane(s, b), e_b = __builtin_amdgcn_readlane(e, b);
                    const float w_b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), b));
                    for (uint32_t pos = s_b + lane; pos < e_b; pos += kWave) val[pos - c0] = w_b;
                }
                {   // short groups, one lane each: as many rounds as the longest of them needs (8, 16 or 32)
                    const uint32_t mine = len <= kGemvExpShort ? len : 0u;
                    const uint32_t rounds = __ballot(mine > 16u) ? 32u : (__ballot(mine > 8u) ? 16u : 8u);
                    for (uint32_t k0 = 0; k0 < rounds; k0 += 8) {
#pragma unroll
                        for (uint32_t k = 0; k < 8; ++k)
                            if (k0 + k < mine) val[s - c0 + k0 + k] = w;
                    }
                }
                const uint32_t done = (uint32_t)__popcll(__ballot(gt + lane < g1 && p.e <= c1));
                gcur = gt + done;
                return done == (uint32_t)kWave && gcur < g1;
            };
            bool more = gcur < g1;
            if (c0 == rs) {  // the first chunk starts at the row's first group: the prefetched tiles apply
#pragma unroll
                for (int t = 0; t < kPre; ++t)
                    if (more) more = expand_tile(pre[t], g0 + (uint32_t)t * kWave);
            }
            while (more) more = expand_tile(load_ptr_tile(v, cser, g0, gcur, g1, lane), gcur);
            wave_lds_sync();
#pragma unroll
            for (uint32_t w = 0; w < NW; ++w)
                if (w < nwin) acc = fmaf(xs[ix[w]], val[w * kWave + lane], acc);
            wave_lds_sync();  // the next chunk overwrites the values
        }
        const float y = wave_sum(acc);
        if (lane == 0) Y[r] = y + t_off;
    }
}

// ------------------------------------------------------------------------------------------------
// batch > 1 with the input tile resident in LDS (reuse of the input, Section V-C)
// ------------------------------------------------------------------------------------------------
//
// The paper finds that loading input elements dominates its AlexNet run and names reuse of the
// input as the remedy.  Here a workgroup of 16 waves copies a tile of V batch columns of ALL n input
// rows into LDS once (n.V.4 bytes: V = 4 up to n = 10000, V = 8 up to n = 5000) and then serves
// the gathers of many rows of W from it.  Lane l of a wave instruction owns colI position w0 + l
// and V columns, as in the batch-1 kernel.  Each wave walks the colI stream of `rpw` CONSECUTIVE
// rows as one stream: the window that holds a row's end is applied twice, once to finish that row
// and once, under the next row's cursor, to start the next one, so the index loads and gathers
// never drain at a row boundary.  The group pointers of the wave's rows are copied to LDS in the
// prologue; a row's list (end, value - Omega[0]) is one pointer per lane, kept in two registers.
// In a window that holds group boundaries every lane multiplies its own input by its own group's
// value (a fused multiply-add costs what an add costs); windows without a boundary only add.
// Needs at most 63 groups per row and K <= 64; X is repacked tile-major by a small kernel first.

constexpr int kXtWaves = 16;

// Xp[t][c][v] = X[c][t.V + v], zero beyond L.  Block (bx, by): input rows 64.bx .. +64 (one per lane),
// tiles 16.by .. +16 spread over the 4 waves: a wave writes 64.V consecutive floats per tile.
template <int V>
__global__ __launch_bounds__(256) void xtile_pack_kernel(const float* __restrict__ X, uint32_t n, uint32_t L, uint32_t ntiles,
                                                         int vec_ok, float* __restrict__ Xp) {
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint32_t c = blockIdx.x * 64u + lane;
    if (c >= n) return;
    const uint32_t t_end = min(ntiles, (blockIdx.y + 1u) * 16u);
    for (uint32_t t = blockIdx.y * 16u + wave; t < t_end; t += 4) {
        const uint32_t col = t * V;
        float4* dst = reinterpret_cast<float4*>(Xp + ((size_t)t * n + c) * V);
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
            const uint32_t cq = col + 4u * q;
            float4 o;
            if (vec_ok && cq + 3u < L) {
                o = *reinterpret_cast<const float4*>(X + (size_t)c * L + cq);
            } else {
                const float* src = X + (size_t)c * L;
                o.x = cq < L ? src[cq] : 0.f;
                o.y = cq + 1u < L ? src[cq + 1u] : 0.f;
                o.z = cq + 2u < L ? src[cq + 2u] : 0.f;
                o.w = cq + 3u < L ? src[cq + 3u] : 0.f;
            }
            dst[q] = o;
        }
    }
}

// Cursor over one row's raw groups: lane j of (l_end, l_w) holds group j's end and value.
struct RCursor {
    uint32_t end;
    float w;
    uint32_t l_end;
    float l_w;
    int next;
};

__device__ __forceinline__ void rcursor_advance(RCursor& c) {
    c.end = __builtin_amdgcn_readlane(c.l_end, c.next);
    c.w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.l_w), c.next));
    ++c.next;
}

// One window of 64 consecutive colI positions starting at w0; this lane's inputs x belong to
// position w0 + who.  A group that ends at or before the window's end is closed here.
template <int V>
__device__ __forceinline__ void xt_step(const float (&x)[V], uint32_t who, uint32_t w0, RCursor& c, float (&run)[V],
                                        float (&acc)[V]) {
    if (__builtin_expect(c.end - w0 > (uint32_t)kWave, 1)) {
#pragma unroll
        for (int k = 0; k < V; ++k) run[k] += x[k];
        return;
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        acc[k] = fmaf(run[k], c.w, acc[k]);  // the sum gathered in earlier windows, times its group's value
        run[k] = 0.f;
    }
    float wl = c.w;
    do {
        const uint32_t lo = c.end - w0;
        rcursor_advance(c);
        wl = who >= lo ? c.w : wl;
    } while (c.end - w0 <= (uint32_t)kWave);
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = fmaf(x[k], wl, acc[k]);
}

// Sum of a[] over the 64 lanes and store of the row's V outputs.  Each of the first log2(V)
// exchange steps halves the components a lane carries; the rest are plain butterfly adds.
template <int V>
__device__ __forceinline__ void xt_store_row(float (&a)[V], uint32_t lane, float* __restrict__ yrow, uint32_t ncols,
                                             const float* __restrict__ Tcol, float omega0) {
    uint32_t comp = 0;
#pragma unroll
    for (int h = V / 2, off = 1; h >= 1; h >>= 1, off <<= 1) {
        const bool up = (lane & (uint32_t)off) != 0;
        comp |= up ? (uint32_t)h : 0u;
#pragma unroll
        for (int k = 0; k < h; ++k) {
            const float keep = up ? a[k + h] : a[k];
            const float give = up ? a[k] : a[k + h];
            a[k] = keep + __shfl_xor(give, off, kWave);
        }
    }
#pragma unroll
    for (int off = V; off < kWave; off <<= 1) a[0] += __shfl_xor(a[0], off, kWave);
    if (lane < (uint32_t)V && comp < ncols) {
        float y = a[0];
        if (omega0 != 0.f) y = fmaf(omega0, Tcol[comp], y);
        yrow[comp] = y;
    }
}

template <int V>
__device__ __forceinline__ void xt_gather(float (&x)[V], const float* xs, uint32_t idx) {
    const float4* p = reinterpret_cast<const float4*>(xs + (size_t)idx * V);
#pragma unroll
    for (int q = 0; q < V / 4; ++q) {
        const float4 t = p[q];
        x[4 * q] = t.x;
        x[4 * q + 1] = t.y;
        x[4 * q + 2] = t.z;
        x[4 * q + 3] = t.w;
    }
}

template <typename IdxT, int V, int U, bool kCser>
__global__ __launch_bounds__(kXtWaves* kWave) void cer_xtile_kernel(KView v, const float* __restrict__ Xp,
                                                                   float* __restrict__ Y, const float* __restrict__ T,
                                                                   uint32_t L, uint32_t ntiles, uint32_t rpw, uint32_t pcap,
                                                                   uint32_t raw_x) {
    extern __shared__ __align__(16) unsigned char xt_smem[];
    constexpr uint32_t SU = U * kWave;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t tile = blockIdx.x % ntiles, rb = blockIdx.x / ntiles;
    const uint32_t xfloats = v.n * V;
    float* xs = reinterpret_cast<float*>(xt_smem);
    uint32_t* wptr = reinterpret_cast<uint32_t*>(xt_smem + (size_t)xfloats * 4) + (size_t)wave * pcap;
    uint8_t* wrank = xt_smem + (size_t)xfloats * 4 + (size_t)kXtWaves * pcap * 4 + (size_t)wave * pcap;

    // this wave's rows and their descriptors, one per lane
    const uint32_t r_begin = min(v.m, (rb * kXtWaves + wave) * rpw), r_end = min(v.m, r_begin + rpw);
    const uint32_t nrows = r_end - r_begin;
    const uint2 info = v.rowInfo[min(r_begin + lane, r_end)];
    if (raw_x) {
        // Xp is the caller's X, [n][L] row-major with L <= V (one tile): widened to V columns on the way in
        for (uint32_t i = threadIdx.x; i < xfloats; i += kXtWaves * kWave) {
            const uint32_t c = i / V, col = i % V;
            xs[i] = col < L ? Xp[(size_t)c * L + col] : 0.f;
        }
    } else {  // the input tile: one contiguous piece of Xp
        const float4* src = reinterpret_cast<const float4*>(Xp + (size_t)tile * xfloats);
        float4* dst = reinterpret_cast<float4*>(xs);
        for (uint32_t i = threadIdx.x; i < xfloats / 4; i += kXtWaves * kWave) dst[i] = src[i];
    }
    const float om_l = v.omega[lane < v.K ? lane : 0u];
    const uint32_t gA = __builtin_amdgcn_readlane(info.x, 0), S0 = __builtin_amdgcn_readlane(info.y, 0);
    const uint32_t gB = __builtin_amdgcn_readlane(info.x, nrows);
    const uint32_t np = gB - gA + 1u;  // at most pcap: the launcher sized it for rpw rows of the fullest kind
    for (uint32_t t = lane; t < np; t += kWave) wptr[t] = v.omegaPtr[gA + t];
    if (kCser)
        for (uint32_t t = lane; t + 1u < np; t += kWave) wrank[t] = (uint8_t)load_rank(v.omegaI, v.omegaI_bits, gA + t);
    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    uint32_t ia[U], ib[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ia[u] = (uint32_t)colI[S0 + u * kWave + lane];
#pragma unroll
    for (int u = 0; u < U; ++u) ib[u] = (uint32_t)colI[S0 + (U + u) * kWave + lane];
    __syncthreads();
    if (nrows == 0) return;

    const float wcer = __shfl(om_l, (int)((lane + 1u) & 63u), kWave) - v.omega0;  // CER: group j of a row has rank j + 1
    RCursor cur;
    uint32_t i = 0, re = 0;
    float acc[V], run[V];
    const uint32_t col0 = tile * V, ncols = min((uint32_t)V, L - col0);
    const float* Tc = T ? T + col0 : nullptr;
    // (re)starts the cursor at row i: a first pseudo group [window start, row start) of weight 0, then the row's groups
#define CER_XT_START(row_start)                                                                          \
    {                                                                                                    \
        const uint32_t g0_ = __builtin_amdgcn_readlane(info.x, i), g1_ = __builtin_amdgcn_readlane(info.x, i + 1); \
        const bool in_ = lane < g1_ - g0_;                                                               \
        const uint32_t t_ = g0_ - gA + (in_ ? lane : 0u);                                                \
        const uint32_t e_ = wptr[t_ + (in_ ? 1u : 0u)];                                                  \
        float w_ = wcer;                                                                                 \
        if (kCser) w_ = __shfl(om_l, (int)wrank[t_], kWave) - v.omega0;                                  \
        cur.l_end = in_ ? e_ : kNoEnd;                                                                   \
        cur.l_w = in_ ? w_ : 0.f;                                                                        \
        cur.end = (row_start);                                                                           \
        cur.w = 0.f;                                                                                     \
        cur.next = 0;                                                                                    \
        re = __builtin_amdgcn_readlane(info.y, i + 1);                                                   \
        _Pragma("unroll") for (int k = 0; k < V; ++k) acc[k] = run[k] = 0.f;                             \
    }
    CER_XT_START(S0)

    float xa[U][V], xb[U][V];
#define CER_XT_LOAD(ix, b) _Pragma("unroll") for (int u = 0; u < U; ++u) ix[u] = (uint32_t)colI[(b) + u * kWave + lane];
#define CER_XT_GATHER(xv, ix) _Pragma("unroll") for (int u = 0; u < U; ++u) xt_gather<V>(xv[u], xs, ix[u]);
#define CER_XT_CONSUME(xv, b)                                                                            \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                      \
        const uint32_t w0_ = (b) + u * kWave;                                                            \
        xt_step<V>(xv[u], lane, w0_, cur, run, acc);                                                     \
        while (re <= w0_ + (uint32_t)kWave) { /* the row ends inside this window */                      \
            xt_store_row<V>(acc, lane, Y + (size_t)(r_begin + i) * L + col0, ncols, Tc, v.omega0);       \
            if (++i == nrows) return;                                                                    \
            CER_XT_START(re)                                                                             \
            xt_step<V>(xv[u], lane, w0_, cur, run, acc);                                                 \
        }                                                                                                \
    }
    CER_XT_GATHER(xa, ia)
    for (uint32_t base = S0;; base += 2 * SU) {
        CER_XT_GATHER(xb, ib)
        CER_XT_LOAD(ia, base + 2 * SU)
        CER_XT_CONSUME(xa, base)
        CER_XT_GATHER(xa, ia)
        CER_XT_LOAD(ib, base + 3 * SU)
        CER_XT_CONSUME(xb, base + SU)
    }
#undef CER_XT_START
#undef CER_XT_LOAD
#undef CER_XT_GATHER
#undef CER_XT_CONSUME
}

// ------------------------------------------------------------------------------------------------
// Column sums of X (Appendix A-A1): T[l] = sum_i X[i,l], in two stages of short partial sums.
// ------------------------------------------------------------------------------------------------

// block (bx, by): columns [bx*CB, +CB), rows [by*slab, +slab).  CB divides 256.
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ X, uint32_t n, uint32_t L,
                                                             uint32_t CB, uint32_t slab, float* __restrict__ part) {
    __shared__ float red[256];
    const uint32_t cl = threadIdx.x % CB, rl = threadIdx.x / CB, RPB = 256u / CB;
    const uint32_t col = blockIdx.x * CB + cl;
    const uint32_t i0 = blockIdx.y * slab, i1 = min(n, i0 + slab);
    float a0 = 0.f, a1 = 0.f;
    if (col < L) {
        uint32_t i = i0 + rl;
        for (; i + RPB < i1; i += 2 * RPB) {
            a0 += X[(size_t)i * L + col];
            a1 += X[(size_t)(i + RPB) * L + col];
        }
        if (i < i1) a0 += X[(size_t)i * L + col];
    }
    red[threadIdx.x] = a0 + a1;
    __syncthreads();
    for (uint32_t s = RPB >> 1; s > 0; s >>= 1) {
        if (rl < s) red[threadIdx.x] += red[threadIdx.x + s * CB];
        __syncthreads();
    }
    if (rl == 0 && col < L) part[(size_t)blockIdx.y * L + col] = red[cl];
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, uint32_t nslabs, uint32_t L,
                                                           float* __restrict__ T) {
    const uint32_t col = blockIdx.x * 256u + threadIdx.x;
    if (col >= L) return;
    float a0 = 0.f, a1 = 0.f;
    uint32_t s = 0;
    for (; s + 1 < nslabs; s += 2) {
        a0 += part[(size_t)s * L + col];
        a1 += part[(size_t)(s + 1) * L + col];
    }
    if (s < nslabs) a0 += part[(size_t)s * L + col];
    T[col] = a0 + a1;
}

// ------------------------------------------------------------------------------------------------
// Launch logic
// ------------------------------------------------------------------------------------------------

struct DeviceInfo {
    int cus = 256;
    size_t lds_per_block = 64 * 1024;
};

const DeviceInfo& device_info() {
    static DeviceInfo info[16];
    static std::once_flag once[16];
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 16) dev = 0;
    std::call_once(once[dev], [dev] {
        hipDeviceProp_t p;
        if (hipGetDeviceProperties(&p, dev) == hipSuccess) {
            info[dev].cus = p.multiProcessorCount > 0 ? p.multiProcessorCount : 256;
            info[dev].lds_per_block = p.sharedMemPerBlock;
            if (p.maxSharedMemoryPerMultiProcessor > info[dev].lds_per_block)
                info[dev].lds_per_block = p.maxSharedMemoryPerMultiProcessor;
        }
    });
    return info[dev];
}

KView make_kview(const DeviceView& d) {
    KView k;
    k.colI = d.colI;
    k.omegaPtr = d.omegaPtr;
    k.rowPtr = d.rowPtr;
    k.rowInfo = static_cast<const uint2*>(d.rowInfo);
    k.omegaI = d.omegaI;
    k.omega = d.omega;
    k.K = (uint32_t)d.K;
    k.omegaI_bits = d.omegaI_bits;
    k.cser = d.cser;
    k.m = (uint32_t)d.m;
    k.n = (uint32_t)d.n;
    k.omega0 = d.omega0;
    return k;
}

int env_int(const char* name, int fallback) {
    const char* s = std::getenv(name);
    return (s && *s) ? std::atoi(s) : fallback;
}

// LDS the batch-1 kernel may claim dynamically: the device's limit less its few static words.
size_t gemv_lds_budget() { return device_info().lds_per_block - 256; }

// Whether the batch-1 kernel stages X in LDS for this matrix: whenever it fits beside Omega and the group lists of
// 4 waves (with at least 64 entries each).
bool gemv_stages_x(const KView& k, uint32_t max_row_groups) {
    const size_t x_bytes = (((size_t)k.n + 3) & ~(size_t)3) * sizeof(float);
    const size_t om_bytes = k.K <= 4096 ? (((size_t)k.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    const uint32_t gcap = std::max<uint32_t>(1u, std::min<uint32_t>(max_row_groups, 1022u));
    return env_int("CER_GEMV_X_GLOBAL", 0) == 0 &&
           x_bytes + om_bytes + (size_t)4 * (std::min<uint32_t>(gcap, 64u) + 2) * 8 <= gemv_lds_budget();
}

template <typename IdxT>
hipError_t launch_gemv(const KView& k, uint32_t max_row_groups, const float* X, float* Y, const float* T,
                       hipStream_t stream) {
    const DeviceInfo& di = device_info();
    const size_t budget = gemv_lds_budget();
    const size_t x_bytes = (((size_t)k.n + 3) & ~(size_t)3) * sizeof(float);
    const bool omega_in_lds = k.K <= 4096;
    const size_t om_bytes = omega_in_lds ? (((size_t)k.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    // per-wave list of non-empty groups: as long as the longest row needs, at most 1022 entries
    uint32_t gcap = std::max<uint32_t>(1u, std::min<uint32_t>(max_row_groups, 1022u));
    auto list_bytes = [&](int waves) { return (size_t)waves * (gcap + 2) * 8; };
    const bool x_in_lds = gemv_stages_x(k, max_row_groups);
    const size_t fixed = (x_in_lds ? x_bytes : 0) + om_bytes;
    // a workgroup that stages a large X should own many rows: 16 waves; small X: 4 waves, more workgroups
    int waves = (x_in_lds && x_bytes > 40 * 1024) ? 16 : 4;
    waves = env_int("CER_GEMV_WAVES", waves);
    if (waves < 1 || waves > 16) return hipErrorInvalidValue;
    while (fixed + list_bytes(waves) > budget && waves > 4) waves >>= 1;
    while (fixed + list_bytes(waves) > budget && gcap > 64) gcap = std::max<uint32_t>(64u, gcap / 2);
    const size_t lds = fixed + list_bytes(waves);
    if (lds > budget) return hipErrorInvalidValue;
    // resident workgroups per CU, limited by LDS and by 32 waves per CU
    size_t per_cu = std::min<size_t>(di.lds_per_block / (lds + 256), (size_t)(32 / waves));
    per_cu = std::max<size_t>(1, std::min<size_t>(per_cu, 8));
    const uint64_t slots = (uint64_t)di.cus * per_cu;
    uint32_t iters = (uint32_t)((k.m + slots * waves - 1) / (slots * waves));
    iters = (uint32_t)env_int("CER_GEMV_ROW_ITERS", (int)std::max<uint32_t>(iters, 1));
    const uint32_t rows_per_block = std::max<uint32_t>(iters, 1) * waves;
    const uint32_t blocks = (k.m + rows_per_block - 1) / rows_per_block;
    const bool vec4 = (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && k.n >= 4;
    using Kern = void (*)(KView, const float*, float*, const float*, uint32_t, int, uint32_t);
    Kern kern;
    const bool few = gcap <= 62 && k.K <= 64;  // gcap is still the longest row's number of groups here
    const bool one = few && rows_per_block == (uint32_t)waves;  // a wave has at most one row
#define CER_GEMV_PICK(CSER, FEW, ONE)                                                            \
    (x_in_lds ? (vec4 ? cer_gemv_kernel<IdxT, true, true, CSER, FEW, ONE>                        \
                      : cer_gemv_kernel<IdxT, true, false, CSER, FEW, ONE>)                      \
              : cer_gemv_kernel<IdxT, false, false, CSER, FEW, ONE>)
    if (k.cser)
        kern = one ? CER_GEMV_PICK(true, true, true) : few ? CER_GEMV_PICK(true, true, false) : CER_GEMV_PICK(true, false, false);
    else
        kern = one ? CER_GEMV_PICK(false, true, true) : few ? CER_GEMV_PICK(false, true, false) : CER_GEMV_PICK(false, false, false);
#undef CER_GEMV_PICK
    const int kslot = (x_in_lds ? (vec4 ? 2 : 1) : 0) + (k.cser ? 3 : 0) + (few ? 6 : 0) + (one ? 6 : 0);
    if (lds > 48 * 1024) {
        // raise the kernel's dynamic-LDS limit once per (kernel, device)
        static std::mutex mu;
        static bool granted[18][16] = {};
        int dev = 0;
        (void)hipGetDevice(&dev);
        dev = (dev >= 0 && dev < 16) ? dev : 0;
        std::lock_guard<std::mutex> lock(mu);
        if (!granted[kslot][dev]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)budget);
            if (e != hipSuccess) return e;
            granted[kslot][dev] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, stream, k, X, Y, T, rows_per_block,
                       omega_in_lds ? 1 : 0, gcap);
    return hipGetLastError();
}

// Launch shape of the batch-1 expansion kernel; waves == 0: X, Omega and the value arrays of four waves do not fit in LDS.
struct GemvExpandPlan {
    int waves = 0;
    uint32_t chunk = 2048;
    size_t lds = 0;
    bool omega_in_lds = false;
};

GemvExpandPlan plan_gemv_expand(const DeviceView& d, const KView& k) {
    GemvExpandPlan p;
    const size_t budget = gemv_lds_budget();
    const size_t x_bytes = (((size_t)k.n + 3) & ~(size_t)3) * sizeof(float);
    p.omega_in_lds = k.K <= 4096;
    const size_t om_bytes = p.omega_in_lds ? (((size_t)k.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    p.chunk = d.nnz <= d.m * 384 ? 512u : 2048u;  // by the average row
    const size_t per_wave = (p.chunk + kWave) * sizeof(float);
    // a workgroup that stages a large X should own many rows; a small X leaves room for more, smaller workgroups
    int waves = x_bytes > 40 * 1024 ? 16 : (k.m >= 8192 ? 16 : (k.m >= 4096 ? 8 : 4));
    while (waves > 4 && x_bytes + om_bytes + waves * per_wave > budget) waves >>= 1;
    if (x_bytes + om_bytes + waves * per_wave > budget) return p;
    p.waves = waves;
    p.lds = x_bytes + om_bytes + waves * per_wave;
    return p;
}

// Rows of short groups go to the expansion kernel.  Measured on 2048 x 2048 matrices, cursor kernel / expansion
// kernel, by indices per non-empty group: 4 (256 values, 50 % zeros) 24.2 / 7.8 us; 1.5 (256 values, 90 %) 16.4 /
// 6.3 us; 16 (64 values, 50 %) 9.4 / 6.6 us; 3 (64 values, 90 %) 8.5 / 5.4 us; 41 (16 values, 70 %) 6.7 / 7.5 us;
// 68 (16 values, 50 %) 6.7 / 8.1 us; AlexNet-fc6 shape (45) 10.2 / 10.5 us; VGG-fc6 shape (90) 8.5 / 16.4 us.
// Short rows (a few hundred indices at most) go there as well: the cursor kernel requests 24 windows of indices per
// row whatever its length (16384 x 512 matrices: 11 - 12 us against 7 - 8 us).
bool gemv_expand_pays(const DeviceView& d) {
    const double per_group = (double)d.nnz / (double)std::max<int64_t>(d.nonempty_groups, 1);
    return per_group < 30.0 || d.nnz <= d.m * 384;
}

// The batch-1 expansion kernel's plan for this matrix if cer_matmul would use it (waves == 0 otherwise).
// CER_GEMV_EXPAND: 1 = whenever X fits in LDS, 0 = never, unset = for rows of short groups.
GemvExpandPlan gemv_expand_choice(const DeviceView& d, const KView& k) {
    const int mode = env_int("CER_GEMV_EXPAND", -1);
    if (mode == 1 || (mode != 0 && gemv_expand_pays(d))) return plan_gemv_expand(d, k);
    return GemvExpandPlan{};
}

template <typename IdxT>
hipError_t launch_gemv_expand(const KView& k, const GemvExpandPlan& p, const float* X, float* Y, hipStream_t stream) {
    using Kern = void (*)(KView, const float*, float*, uint32_t, int);
    const bool small = p.chunk == 512;
    Kern kern = k.cser ? (small ? cer_gemv_expand_kernel<IdxT, true, 512> : cer_gemv_expand_kernel<IdxT, true, 2048>)
                       : (small ? cer_gemv_expand_kernel<IdxT, false, 512> : cer_gemv_expand_kernel<IdxT, false, 2048>);
    if (p.lds > 48 * 1024) {
        static std::mutex mu;
        static bool granted[4][16] = {};
        const int slot = (k.cser ? 1 : 0) + (small ? 2 : 0);
        int dev = 0;
        (void)hipGetDevice(&dev);
        dev = (dev >= 0 && dev < 16) ? dev : 0;
        std::lock_guard<std::mutex> lock(mu);
        if (!granted[slot][dev]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)gemv_lds_budget());
            if (e != hipSuccess) return e;
            granted[slot][dev] = true;
        }
    }
    const uint32_t rows_per_block = (uint32_t)p.waves;
    const uint32_t blocks = (k.m + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(p.waves * kWave), p.lds, stream, k, X, Y, rows_per_block,
                       p.omega_in_lds ? 1 : 0);
    return hipGetLastError();
}

// The kernel that expands the group values per position is the default: measured on MI355X it beats the cursor
// kernel on every workload (1.05 - 1.2 x on the layer shapes, up to 2 x on rows of many short groups).
// CER_GEMM_EXPAND=0 selects the cursor kernel.
// The default kernel on a matrix with rows of unequal length: one wave per (batch tile, further part of a long row)
// writing into a stream-ordered temporary, then the ordinary work list in descending order of row length, then the
// kernel that adds the parts' sums to Y.
template <typename Kern>
hipError_t launch_expand_split(Kern kern, const KView& k, const float* X, float* Y, const float* T, uint32_t L,
                               uint32_t ntiles, uint32_t rowblocks, uint32_t ipx, SplitArgs sp, hipStream_t stream) {
    const uint64_t part_blocks = ((((uint64_t)ntiles * sp.nparts + 3) / 4) + 7) & ~(uint64_t)7;
    const uint64_t blocks = (uint64_t)ipx * 8 + part_blocks;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    float* out = nullptr;
    hipError_t e = hipSuccess;
    if (sp.nparts > 0) {
        e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&out), (size_t)sp.nparts * L * sizeof(float), stream);
        if (e != hipSuccess) return e;
    }
    sp.out = out;
    sp.part_blocks = (uint32_t)part_blocks;
    hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(256), 0, stream, k, X, Y, T, L, ntiles, rowblocks, ipx, sp);
    e = hipGetLastError();
    if (sp.nparts > 0) {
        if (e == hipSuccess) {
            hipLaunchKernelGGL(split_add_kernel, dim3(sp.nrows), dim3(256), 0, stream, sp.rows, out, Y, L);
            e = hipGetLastError();
        }
        const hipError_t f = (hipError_t)temp_free(out, stream);
        if (e == hipSuccess) e = f;
    }
    return e;
}

template <typename IdxT, int V, int P>
hipError_t launch_gemm_vp(const KView& k, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                          const SplitArgs& sp, bool short_rows = false) {
    constexpr uint32_t TW = V * P;
    const uint32_t ntiles = (L + TW - 1) / TW;
    const uint32_t rowblocks = (k.m + 3) / 4;
    const uint64_t nitems = (uint64_t)ntiles * rowblocks;
    if (nitems > 0x7FFFFFFFull / 8) return hipErrorInvalidValue;
    const uint32_t ipx = (uint32_t)((nitems + 7) / 8);
    if (env_int("CER_GEMM_EXPAND", 1) != 0) {
        if (sp.order) {
            if (TW == 32 && V == 4 && short_rows)
                return launch_expand_split(cer_gemm_expand_kernel<IdxT, 4, 8, false, kExpChunkShort, true>, k, X, Y, T, L,
                                           ntiles, rowblocks, ipx, sp, stream);
            return launch_expand_split(cer_gemm_expand_kernel<IdxT, V, P, false, kExpChunkLong, true>, k, X, Y, T, L, ntiles,
                                       rowblocks, ipx, sp, stream);
        }
        if (TW == 32 && V == 4 && short_rows)
            hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, 8, false, kExpChunkShort>), dim3(ipx * 8), dim3(256), 0, stream,
                               k, X, Y, T, L, ntiles, rowblocks, ipx, SplitArgs{});
        else
            hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, V, P, false>), dim3(ipx * 8), dim3(256), 0, stream, k, X, Y, T, L,
                               ntiles, rowblocks, ipx, SplitArgs{});
    } else
        hipLaunchKernelGGL((cer_gemm_kernel<IdxT, V, P>), dim3(ipx * 8), dim3(256), 0, stream, k, X, Y, T, L, ntiles,
                           rowblocks, ipx);
    return hipGetLastError();
}

// The default kernel on a batch whose width is not a multiple of 4, or whose X / Y are only 4-byte aligned (L >= 4).
template <typename IdxT, int P>
hipError_t launch_gemm_ragged(const KView& k, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                              const SplitArgs& sp, bool short_rows = false) {
    constexpr uint32_t TW = 4 * P;
    const uint32_t ntiles = (L + TW - 1) / TW;
    const uint32_t rowblocks = (k.m + 3) / 4;
    const uint64_t nitems = (uint64_t)ntiles * rowblocks;
    if (nitems > 0x7FFFFFFFull / 8 || L < 4) return hipErrorInvalidValue;
    const uint32_t ipx = (uint32_t)((nitems + 7) / 8);
    if (sp.order) {
        if (P == 8 && short_rows)
            return launch_expand_split(cer_gemm_expand_kernel<IdxT, 4, 8, true, kExpChunkShort, true>, k, X, Y, T, L, ntiles,
                                       rowblocks, ipx, sp, stream);
        return launch_expand_split(cer_gemm_expand_kernel<IdxT, 4, P, true, kExpChunkLong, true>, k, X, Y, T, L, ntiles,
                                   rowblocks, ipx, sp, stream);
    }
    if (P == 8 && short_rows)
        hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, 8, true, kExpChunkShort>), dim3(ipx * 8), dim3(256), 0, stream, k, X,
                           Y, T, L, ntiles, rowblocks, ipx, SplitArgs{});
    else
        hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, P, true>), dim3(ipx * 8), dim3(256), 0, stream, k, X, Y, T, L,
                           ntiles, rowblocks, ipx, SplitArgs{});
    return hipGetLastError();
}

inline uint32_t pow2_ceil(uint32_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Tile width (32, 64 or 128 batch columns) for a batch wider than 32 columns.  A gather instruction costs what the
// cache lines it touches cost: when a row of X is a whole number of 128-byte lines, 32-column tiles touch exactly the
// lines they need; otherwise every piece of a row touches up to one line more than its width, and wider tiles mean
// fewer pieces.  Against that stand the lanes a wide tile leaves idle on a narrow batch and the waves it leaves
// unlaunched on a matrix of few rows.  Measured on MI355X (AlexNet-fc6 shape, 32 / 64 / 128 columns per tile):
// batch 96: 91 / 115 / 107 us; batch 100: 186 / 145 / 120 us; batch 40: 99 / 67 / 105 us; 3x3 convolution shape,
// batch 100 (512 rows): 35 / 30 / 44 us.
uint32_t pick_wide_tile(uint32_t L, uint32_t m, const float* X, uint32_t max_tile) {
    const uint32_t row_bytes = L * 4u, base = (uint32_t)(reinterpret_cast<uintptr_t>(X) & 127u);
    const uint32_t step = std::gcd(row_bytes, 128u);  // rows start at base + multiples of this within a line
    auto lines = [&](uint32_t offset, uint32_t bytes) {  // average number of lines a piece of a row touches
        double sum = 0;
        uint32_t cnt = 0;
        for (uint32_t ph = 0; ph < 128u; ph += step, ++cnt) sum += (double)(((base + ph + offset) % 128u + bytes + 127u) / 128u);
        return sum / cnt;
    };
    uint32_t best_tile = 32;
    double best = 1e300;
    for (uint32_t tw = 32; tw <= max_tile; tw *= 2) {
        const uint32_t ntiles = (L + tw - 1) / tw, last_cols = L - (ntiles - 1) * tw;
        const double fill = (double)L / ((double)ntiles * tw);
        const double waves = (double)m * ntiles;
        double cost = (ntiles - 1) * lines(0, tw * 4u) + lines(((ntiles - 1) * tw * 4u) % 128u, last_cols * 4u);
        cost *= std::max(1.0, 0.62 / fill) / std::min(1.0, waves / 1024.0);
        if (cost < 0.95 * best) {
            best = cost;
            best_tile = tw;
        }
    }
    return best_tile;
}

template <typename IdxT>
hipError_t launch_gemm(const KView& k, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                       const SplitArgs& sp, bool short_rows) {
    const bool vec4 = (L % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0) &&
                      ((reinterpret_cast<uintptr_t>(Y) & 15u) == 0) && ((reinterpret_cast<uintptr_t>(T) & 15u) == 0);
    if (vec4) {
        // tile width: all of L up to 32 columns, 32 beyond: one gather = one 128-byte line of an X row, and a
        // wider batch gives more waves (measured on MI355X: 32 beats 16, 64, 128 and 256 at L = 32, 64, 3136)
        uint32_t tw = std::min<uint32_t>(pow2_ceil(L), 32u);
        tw = std::max<uint32_t>(tw, 8u);  // 4-column tiles (64 distinct rows per gather instruction) measured 1.4 - 3 x slower
        if (L > 32) tw = pick_wide_tile(L, k.m, X, 128u);
        tw = (uint32_t)env_int("CER_GEMM_TILE", (int)tw);
        switch (tw) {
            case 4: return launch_gemm_vp<IdxT, 4, 1>(k, X, Y, T, L, stream, sp);
            case 8: return launch_gemm_vp<IdxT, 4, 2>(k, X, Y, T, L, stream, sp);
            case 16: return launch_gemm_vp<IdxT, 4, 4>(k, X, Y, T, L, stream, sp);
            case 32: return launch_gemm_vp<IdxT, 4, 8>(k, X, Y, T, L, stream, sp, short_rows);
            case 64: return launch_gemm_vp<IdxT, 4, 16>(k, X, Y, T, L, stream, sp);
            case 128: return launch_gemm_vp<IdxT, 4, 32>(k, X, Y, T, L, stream, sp);
            case 256: return launch_gemm_vp<IdxT, 4, 64>(k, X, Y, T, L, stream, sp);
            default: return hipErrorInvalidValue;
        }
    }
    if (L >= 4 && env_int("CER_GEMM_EXPAND", 1) != 0 && env_int("CER_GEMM_RAGGED", 1) != 0) {
        // ragged width or 4-byte aligned buffers: still four columns per lane (CER_GEMM_RAGGED=0: one column per lane)
        uint32_t rtw = std::max<uint32_t>(std::min<uint32_t>(pow2_ceil(L), 32u), 8u);
        if (L > 32) rtw = pick_wide_tile(L, k.m, X, 128u);
        switch (rtw) {
            case 8: return launch_gemm_ragged<IdxT, 2>(k, X, Y, T, L, stream, sp);
            case 16: return launch_gemm_ragged<IdxT, 4>(k, X, Y, T, L, stream, sp);
            case 32: return launch_gemm_ragged<IdxT, 8>(k, X, Y, T, L, stream, sp, short_rows);
            case 64: return launch_gemm_ragged<IdxT, 16>(k, X, Y, T, L, stream, sp);
            default: return launch_gemm_ragged<IdxT, 32>(k, X, Y, T, L, stream, sp);
        }
    }
    const uint32_t tw = std::min<uint32_t>(pow2_ceil(L), 64u);
    switch (tw) {
        case 1: case 2: return launch_gemm_vp<IdxT, 1, 2>(k, X, Y, T, L, stream, sp);
        case 4: return launch_gemm_vp<IdxT, 1, 4>(k, X, Y, T, L, stream, sp);
        case 8: return launch_gemm_vp<IdxT, 1, 8>(k, X, Y, T, L, stream, sp);
        case 16: return launch_gemm_vp<IdxT, 1, 16>(k, X, Y, T, L, stream, sp);
        case 32: return launch_gemm_vp<IdxT, 1, 32>(k, X, Y, T, L, stream, sp);
        default: return launch_gemm_vp<IdxT, 1, 64>(k, X, Y, T, L, stream, sp);
    }
}

// Plan of the LDS-resident-input variant; valid == false: not applicable to this matrix / batch.
struct XtilePlan {
    bool valid = false;
    int V = 4;
    uint32_t ntiles = 0, rpw = 1, pcap = 0, blocks = 0;
    size_t lds = 0;
    double est_clk = 0;  // rough duration, for the choice against the L2-gather kernel
};

XtilePlan plan_xtile(const DeviceView& d, uint32_t L) {
    XtilePlan p;
    const DeviceInfo& di = device_info();
    if (L < 2 || d.m < 1 || d.max_row_groups > 63 || d.K > 64 || d.n < 1) return p;
    const uint64_t nnz_avg = (uint64_t)(d.nnz / std::max<int64_t>(d.m, 1)) + 1;
    for (int V : {8, 4}) {
        const size_t xbytes = (size_t)d.n * V * 4;
        if (V == 8 && L < 8) continue;
        const uint32_t ntiles = (L + V - 1) / V;
        if (ntiles > 65535u * 16u) continue;  // grid of the repacking kernel
        double best = 0;
        uint32_t best_rpw = 0;
        for (uint32_t rpw : {1u, 2u, 4u, 8u, 16u, 32u, 63u}) {
            const uint32_t pcap = ((uint32_t)(rpw * d.max_row_groups + 1) + 3u) & ~3u;
            const size_t lds = xbytes + (size_t)kXtWaves * pcap * (d.cser ? 5 : 4);
            if (lds > di.lds_per_block) break;
            const uint64_t rowblocks = ((uint64_t)d.m + (uint64_t)kXtWaves * rpw - 1) / ((uint64_t)kXtWaves * rpw);
            const uint64_t blocks = rowblocks * ntiles;
            if (blocks > 0x7FFFFFFFull) continue;
            const double rounds = (double)((blocks + di.cus - 1) / di.cus);
            // per workgroup: staging at 64 B/clk, then 16 waves on 4 SIMDs, about 4.(V + 12) clocks per window
            const double stage = (double)xbytes / 64.0 + 2000.0;
            const double windows = (double)rpw * ((double)nnz_avg / 64.0 + 2.0);
            const double work = windows * 4.0 * (V + 12) * 4.0;
            const double t = rounds * (stage + work);
            if (best_rpw == 0 || t < best) {
                best = t;
                best_rpw = rpw;
            }
            if (rpw >= (uint32_t)d.m) break;
        }
        if (best_rpw == 0) continue;
        p.valid = true;
        p.V = V;
        p.ntiles = ntiles;
        p.rpw = best_rpw;
        p.pcap = ((uint32_t)(best_rpw * d.max_row_groups + 1) + 3u) & ~3u;
        p.lds = xbytes + (size_t)kXtWaves * p.pcap * (d.cser ? 5 : 4);
        p.blocks = (uint32_t)((((uint64_t)d.m + (uint64_t)kXtWaves * best_rpw - 1) / ((uint64_t)kXtWaves * best_rpw)) * ntiles);
        p.est_clk = best;
        return p;
    }
    return p;
}

// Whether the LDS variant is expected to beat the kernel that gathers from L2.  Measured on MI355X: for wide
// batches it never does -- gathers of 16- or 32-byte pieces at random LDS addresses are bank-conflict bound at
// 32 - 43 B/clk per CU, while the L2 kernel's gathers of whole 128-byte rows sustain 27 - 48 B/clk per CU and
// amortise the group structure over 32 batch columns instead of 4 or 8 (AlexNet-fc6 shape, batch 32: 62 us against
// 35 us; 3x3 convolution shape, batch 3136: 536 us against 378 us).  For narrow batches it does: the L2 kernel
// still moves a whole 128-byte line per index, the LDS kernel 16 or 32 bytes (AlexNet-fc6 shape, batch 2 / 3 / 4 /
// 6 / 8: 28 / 29 / 29 / 37 / 31 us from L2, 23 / 22 / 13 / 28 / 28 us from LDS with the tile-major copy, less
// without it), provided the matrix is large enough for the gathers to dominate the launch (2048 x 2048 cells with
// 0.2 - 2 million indices: 6 - 12 us either way, the L2 kernel ahead).
bool xtile_pays(const XtilePlan& p, const DeviceView& d, uint32_t L) {
    (void)p;
    return L <= 8 && d.nnz >= 2500000;
}

template <typename IdxT, int V, int U>
hipError_t launch_xtile_v(const KView& k, const XtilePlan& p, const float* Xp, uint32_t raw_x, float* Y, const float* T,
                          uint32_t L, hipStream_t stream, int slot) {
    using Kern = void (*)(KView, const float*, float*, const float*, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t);
    Kern kern = k.cser ? cer_xtile_kernel<IdxT, V, U, true> : cer_xtile_kernel<IdxT, V, U, false>;
    slot = slot * 2 + (k.cser ? 1 : 0);
    if (p.lds > 48 * 1024) {
        static std::mutex mu;
        static bool granted[12][16] = {};
        int dev = 0;
        (void)hipGetDevice(&dev);
        dev = (dev >= 0 && dev < 16) ? dev : 0;
        std::lock_guard<std::mutex> lock(mu);
        if (!granted[slot][dev]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)device_info().lds_per_block);
            if (e != hipSuccess) return e;
            granted[slot][dev] = true;
        }
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kXtWaves * kWave), p.lds, stream, k, Xp, Y, T, L, p.ntiles, p.rpw, p.pcap,
                       raw_x);
    return hipGetLastError();
}

template <typename IdxT>
hipError_t launch_xtile(const KView& k, const XtilePlan& p, const float* X, float* Y, const float* T, uint32_t L,
                        hipStream_t stream, int idx_slot) {
    // tile-major copy of X in a stream-ordered temporary; a batch of one tile is staged straight from X
    const float* Xp = X;
    float* tmp = nullptr;
    const bool one_tile = p.ntiles == 1;
    const uint32_t raw_x = one_tile && !(L == (uint32_t)p.V && (reinterpret_cast<uintptr_t>(X) & 15u) == 0) ? 1u : 0u;
    if (!one_tile) {
        hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&tmp), (size_t)p.ntiles * k.n * p.V * sizeof(float), stream);
        if (e != hipSuccess) return e;
        const int vec_ok = (L % 4 == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0) ? 1 : 0;
        const dim3 grid((k.n + 63) / 64, (p.ntiles + 15) / 16);
        if (p.V == 8)
            hipLaunchKernelGGL(xtile_pack_kernel<8>, grid, dim3(256), 0, stream, X, k.n, L, p.ntiles, vec_ok, tmp);
        else
            hipLaunchKernelGGL(xtile_pack_kernel<4>, grid, dim3(256), 0, stream, X, k.n, L, p.ntiles, vec_ok, tmp);
        e = hipGetLastError();
        if (e != hipSuccess) {
            (void)temp_free(tmp, stream);
            return e;
        }
        Xp = tmp;
    }
    hipError_t e = p.V == 8 ? launch_xtile_v<IdxT, 8, 3>(k, p, Xp, raw_x, Y, T, L, stream, idx_slot * 2 + 1)
                            : launch_xtile_v<IdxT, 4, 8>(k, p, Xp, raw_x, Y, T, L, stream, idx_slot * 2);
    if (tmp) {
        hipError_t f = (hipError_t)temp_free(tmp, stream);
        if (e == hipSuccess) e = f;
    }
    return e;
}

hipError_t launch_colsum(const float* X, uint32_t n, uint32_t L, float* part, uint32_t nslabs, uint32_t slab,
                         uint32_t CB, float* T, hipStream_t stream) {
    const uint32_t coltiles = (L + CB - 1) / CB;
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(coltiles, nslabs), dim3(256), 0, stream, X, n, L, CB, slab, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(colsum_final_kernel, dim3((L + 255) / 256), dim3(256), 0, stream, part, nslabs, L, T);
    return hipGetLastError();
}

// Large batches of a matrix that is not sparse enough: the gathers move nnz.4.batch bytes through the L1/L2 path
// (measured 18 - 31 TB/s chip-wide, 24 taken here), the fp32 matrix cores need 2.m.n.batch flops (the dense kernel
// of this library: 12 - 20 us + flops / 90 ... 120 TFLOP/s, rising with the size), so from about one indexed
// element in five upwards the dense contraction is the faster way to the same Y.  The matrix is then decoded into a
// stream-ordered temporary (4.m.n bytes, bounded here; written at about 4.5 TB/s) and multiplied on the matrix
// cores.  Measured on MI355X, gathers against decode + dense: 3x3 convolution shape (60 % zeros) batch 3136
// 391 / 201 us, batch 784 165 / 75 us, batch 256 44 / 45 us; AlexNet-fc6 shape (85 %) batch 2048 1917 / 1466 us,
// batch 512 419 / 421 us; VGG-fc6 shape (95 %) batch 1024 1187 / 2017 us; 2048 x 2048, batch 1024: 70 % zeros
// 187 / 119 us, 80 % 139 / 119 us, 90 % 89 / 118 us.
// Narrow batches of a dense-ish matrix take the same route: a gather moves a whole 128-byte line however narrow the
// batch, so a 4096 x 9216 layer quantized to 7 bits (71 % of the elements indexed) costs 171 us at batch 32 by
// gathers, 70 us decoded (30 us) and multiplied by the dense kernel (40 us, itself bound by reading the matrix).
bool densify_pays(const DeviceView& d, uint32_t L) {
    if (L < 2 || d.m < 128 || d.n < 256) return false;
    const double mn = (double)d.m * (double)d.n;
    if (mn * 4.0 > (double)(1ull << 30)) return false;
    const double flops = 2.0 * mn * L;
    // every (row, tile) is a wave whose start-up chain (descriptor -> pointers -> indices -> first gathers) takes about
    // 4 us, 4096 of them in flight: what bounds matrices of many short rows (16384 x 512: batch 128 64 - 84 us,
    // batch 512 160 - 440 us by gathers; 44 - 49 us and 94 - 103 us decoded and multiplied)
    const double tiles = std::ceil((double)L / 32.0);
    const double t_gather = std::max((double)d.nnz * std::max(4.0 * L, 128.0) / 24e12, (double)d.m * tiles * 4e-6 / 4096.0);
    const double rate = flops < 1.5e10 ? 90e12 : (flops < 1e11 ? 105e12 : 120e12);
    const double t_write = 4.0 * mn / 4.5e12;  // the decoded matrix goes to memory once and is read back at least once
    const double t_decode = t_write + (double)d.nnz * 1.5e-12 + 3e-6;  // measured 30 us (5.7 M indices) ... 88 us (28.7 M)
    const double t_dense = (flops < 5e9 ? 20e-6 : 12e-6) + std::max(flops / rate, t_write) + t_decode;
    return t_gather > 1.1 * t_dense;
}

hipError_t launch_densified(const DeviceView& d, const float* X, float* Y, uint32_t L, hipStream_t stream) {
    float* W = nullptr;
    hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&W), (size_t)d.m * (size_t)d.n * sizeof(float), stream);
    if (e != hipSuccess) return e;
    if (decode_device(d, W, stream) != 0) e = hipErrorLaunchFailure;  // a CER_* code: only a failed launch is possible
    if (e == hipSuccess) e = (hipError_t)launch_dense(W, X, Y, d.m, d.n, (int64_t)L, stream);
    const hipError_t f = (hipError_t)temp_free(W, stream);
    return e == hipSuccess ? f : e;
}

// Which kernel serves a batch of L > 1 columns (cer_matmul_path's numbering: 1, 2 or 3).
//   CER_DENSIFY: 1 = decode + dense product for every batch > 1, 0 = never, unset = by the estimate above
//   CER_XTILE:   1 = input tile in LDS whenever applicable, 0 = never, unset = by estimate (narrow batches)
int choose_batched_path(const DeviceView& d, uint32_t L, XtilePlan* plan_out) {
    const int dense_mode = env_int("CER_DENSIFY", -1), lds_mode = env_int("CER_XTILE", -1);
    const bool has_elements = d.m > 0 && d.n > 0;
    if (dense_mode == 1 && has_elements) return 3;
    const XtilePlan plan = lds_mode == 0 ? XtilePlan{} : plan_xtile(d, L);
    if (plan.valid && (lds_mode == 1 || xtile_pays(plan, d, L))) {
        if (plan_out) *plan_out = plan;
        return 2;
    }
    if (dense_mode != 0 && has_elements && densify_pays(d, L)) return 3;
    return 1;
}

}  // namespace

int matmul_path(const DeviceView& d, int64_t L) {
    if (L <= 1) return gemv_expand_choice(d, make_kview(d)).waves > 0 ? 4 : 0;
    if (L > 0x7FFFFFFFll) return 1;
    return choose_batched_path(d, (uint32_t)L, nullptr);
}

int launch_matmul(const DeviceView& d, const float* X, float* Y, int64_t L64, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (d.m == 0) return (int)hipSuccess;
    if (L64 > 0x7FFFFFFFll || d.m > 0x7FFFFFFFll) return (int)hipErrorInvalidValue;
    const uint32_t L = (uint32_t)L64;
    XtilePlan plan;
    const int batched_path = L > 1 ? choose_batched_path(d, L, &plan) : 0;
    if (batched_path == 3) return (int)launch_densified(d, X, Y, L, stream);
    const KView k = make_kview(d);

    float* T = nullptr;
    float* scratch = nullptr;
    hipError_t e = hipSuccess;
    const GemvExpandPlan gx = L == 1 ? gemv_expand_choice(d, k) : GemvExpandPlan{};
    const bool gemv_sums_x = L == 1 && (gx.waves > 0 || gemv_stages_x(k, (uint32_t)d.max_row_groups));
    if (d.omega0 != 0.f && !gemv_sums_x) {
        // T[l] = sum_i X[i,l] in a stream-ordered temporary: [T: L rounded to 64][partials: nslabs x L]
        const uint32_t CB = std::min<uint32_t>(256u, pow2_ceil(L));
        const uint32_t coltiles = (L + CB - 1) / CB;
        uint32_t nslabs = std::max<uint32_t>(1u, std::min<uint32_t>(((uint32_t)d.n + 255u) / 256u, 1024u / coltiles));
        nslabs = std::max<uint32_t>(nslabs, 1u);
        const uint32_t slab = ((uint32_t)d.n + nslabs - 1) / nslabs;
        const size_t t_floats = ((size_t)L + 63) & ~(size_t)63;
        e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&scratch), (t_floats + (size_t)nslabs * L) * sizeof(float), stream);
        if (e != hipSuccess) return (int)e;
        T = scratch;
        e = launch_colsum(X, (uint32_t)d.n, L, scratch + t_floats, nslabs, std::max<uint32_t>(slab, 1u), CB, T, stream);
        if (e != hipSuccess) {
            (void)temp_free(scratch, stream);
            return (int)e;
        }
    }
    if (L == 1 && gx.waves > 0) {
        switch (d.colI_bits) {
            case 8: e = launch_gemv_expand<uint8_t>(k, gx, X, Y, stream); break;
            case 16: e = launch_gemv_expand<uint16_t>(k, gx, X, Y, stream); break;
            default: e = launch_gemv_expand<uint32_t>(k, gx, X, Y, stream); break;
        }
    } else if (L == 1) {
        switch (d.colI_bits) {
            case 8: e = launch_gemv<uint8_t>(k, (uint32_t)d.max_row_groups, X, Y, T, stream); break;
            case 16: e = launch_gemv<uint16_t>(k, (uint32_t)d.max_row_groups, X, Y, T, stream); break;
            default: e = launch_gemv<uint32_t>(k, (uint32_t)d.max_row_groups, X, Y, T, stream); break;
        }
    } else {
        if (batched_path == 2) {
            switch (d.colI_bits) {
                case 8: e = launch_xtile<uint8_t>(k, plan, X, Y, T, L, stream, 0); break;
                case 16: e = launch_xtile<uint16_t>(k, plan, X, Y, T, L, stream, 1); break;
                default: e = launch_xtile<uint32_t>(k, plan, X, Y, T, L, stream, 2); break;
            }
        } else {
            // CER_GEMM_SHORT: 0 = never the 512-position chunks, 1 = always (32-column tiles), unset = by the average row
            const int sm = env_int("CER_GEMM_SHORT", -1);
            const bool short_rows = sm == 1 || (sm != 0 && d.nnz <= d.m * 384);
            SplitArgs sp;  // CER_GEMM_SPLIT=0: rows in their own order, long rows whole
            if (d.row_order && env_int("CER_GEMM_SPLIT", 1) != 0) {
                sp.order = static_cast<const uint32_t*>(d.row_order);
                sp.parts = static_cast<const uint4*>(d.split_parts);
                sp.rows = static_cast<const uint4*>(d.split_rows);
                sp.nparts = d.n_split_parts;
                sp.nrows = d.n_split_rows;
                sp.len = d.split_len;
                sp.min = d.split_min;
            }
            switch (d.colI_bits) {
                case 8: e = launch_gemm<uint8_t>(k, X, Y, T, L, stream, sp, short_rows); break;
                case 16: e = launch_gemm<uint16_t>(k, X, Y, T, L, stream, sp, short_rows); break;
                default: e = launch_gemm<uint32_t>(k, X, Y, T, L, stream, sp, short_rows); break;
            }
        }
    }
    if (scratch) {
        hipError_t f = (hipError_t)temp_free(scratch, stream);
        if (e == hipSuccess) e = f;
    }
    return (int)e;
}

}  // namespace cer
