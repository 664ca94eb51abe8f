// Shared by the product kernels' translation units (gfx950, wave64): what a kernel sees of a handle, the list of a
// row's non-empty groups and the wave-uniform cursor over it (Algorithms 3 and 4 of the paper mapped onto a
// wavefront), the cross-lane sum, and the launchers' view of the device.
//
// Mapping of the method onto the machine
//   * one wavefront owns one output row (times one tile of batch columns);
//   * the wave first turns the row's group pointers into a compact list of its NON-EMPTY groups
//     in LDS: (end offset into colI, value - Omega[0]).  CER derives the value from the group's
//     position in the row, CSER from OmegaI; empty CER padding groups vanish here (ballot +
//     prefix-popcount compaction), so both formats share every later step;
//   * one wave instruction always covers CONSECUTIVE positions of colI (64 of them for batch 1,
//     64/P for a batch tile handled by P lanes per index), so the group structure is wave-uniform.
// Every load that feeds the streams is unconditional and issued in straight-line code (colI is
// followed by readable padding); positions past a row's end pick up some valid input that is
// multiplied by the weight 0 of the list's sentinel.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cmath>
#include <mutex>
#include <numeric>
#include <type_traits>

#include "cer_internal.hpp"

namespace cer {

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
    const uint32_t* rank_tab;  // derived: the rank table (null: none), 1 << rank_tab_shift words per row
    int32_t rank_tab_shift;
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

// The same for the first tile of a row, which in most matrices is the row's only one and holds fewer than 64 groups:
// one vector-memory instruction for the pointers instead of two (a wave instruction costs the memory pipeline the
// same whatever it fetches) -- a lane's group ends where its right-hand neighbour's begins, so the end comes from
// the neighbour lane (DPP wave_shl:1).  A full tile takes the two independent loads above.
__device__ __forceinline__ PtrTile load_ptr_tile_first(const KView& v, bool cser, uint32_t g0, uint32_t j0, uint32_t tg_end,
                                                 uint32_t lane) {
    if (tg_end > j0 && tg_end - j0 >= (uint32_t)kWave) return load_ptr_tile(v, cser, g0, j0, tg_end, lane);  // wave-uniform
    const uint32_t g = j0 + lane;
    const uint32_t gc = min(g, tg_end);  // lanes past the tile load the tile's end pointer
    PtrTile p;
    p.s = v.omegaPtr[gc];
    p.e = (uint32_t)__builtin_amdgcn_update_dpp((int)p.s, (int)p.s, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
    const uint32_t gr = g < tg_end ? g : (tg_end > j0 ? tg_end - 1u : j0);
    p.rank = cser ? load_rank(v.omegaI, v.omegaI_bits, gr) : gr - g0 + 1u;
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
// Host side: helpers of the launchers, and what the translation units offer each other
// ------------------------------------------------------------------------------------------------

inline KView make_kview(const DeviceView& d) {
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
    k.rank_tab = d.rank_tab;
    k.rank_tab_shift = d.rank_tab_shift;
    return k;
}

inline uint32_t pow2_ceil(uint32_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Raises a kernel's dynamic-LDS limit once per (kernel slot, device); no lock is taken once it is granted.
template <int kSlots>
struct LdsGrant {
    std::atomic<bool> granted[kSlots][16] = {};
    std::mutex mu;
    hipError_t ensure(int slot, const void* kernel, size_t bytes) {
        int dev = 0;
        (void)hipGetDevice(&dev);  // a thread-local read inside the runtime
        dev = (dev >= 0 && dev < 16) ? dev : 0;
        if (granted[slot][dev].load(std::memory_order_acquire)) return hipSuccess;
        std::lock_guard<std::mutex> lock(mu);
        if (!granted[slot][dev].load(std::memory_order_relaxed)) {
            const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            granted[slot][dev].store(true, std::memory_order_release);
        }
        return hipSuccess;
    }
};

// cer_gemv.hip -- batch 1.  gemv_path: 0 (cursor kernel) or 4 (expansion kernel) for this matrix and these options;
// gemv_sums_x: whether that kernel forms Omega[0] . sum_i X[i] itself from its staged copy of X (otherwise the
// launcher passes T = the column sum of X).
int gemv_path(const DeviceView& d, const MatmulOptions& o);
bool gemv_sums_x(const DeviceView& d, const MatmulOptions& o);
hipError_t launch_gemv_any(const DeviceView& d, const float* X, float* Y, const float* T, hipStream_t stream,
                           const MatmulOptions& o);

// cer_gemm.hip -- batch > 1, rows of X gathered from L2 (T: column sums of X when Omega[0] != 0, else unused)
hipError_t launch_gemm_any(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                           const MatmulOptions& o);

// cer_xtile.hip -- batch > 1, a tile of X resident in LDS.  valid == false: not applicable to this matrix / batch.
struct XtilePlan {
    bool valid = false;
    int V = 4;
    uint32_t ntiles = 0, rpw = 1, pcap = 0, blocks = 0;
    size_t lds = 0;
    double est_clk = 0;  // rough duration
};
XtilePlan plan_xtile(const DeviceView& d, uint32_t L);
hipError_t launch_xtile_any(const DeviceView& d, const XtilePlan& p, const float* X, float* Y, const float* T, uint32_t L,
                            hipStream_t stream);

// cer_strip.hip -- batch > 1, strips of X resident in LDS (needs the strip-major index of cer_prepare_strips)
bool strip_applicable(const DeviceView& d, const float* X, const float* Y, uint32_t L);
struct StripPlan {
    uint32_t ntiles = 0, nsplit = 1, rows_per_split = 0;
    uint64_t blocks = 0;
    double est_us = 0;  // rough duration of the two launches
};
StripPlan plan_strip(const DeviceView& d, uint32_t L);
hipError_t launch_strip(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream);

}  // namespace cer
