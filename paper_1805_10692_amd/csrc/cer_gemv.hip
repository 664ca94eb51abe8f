// Batch 1 (one input vector): Y = W.x with W in CER / CSER form (Appendix A-C, Algorithms 3 and 4 of the paper; the
// constant term of a non-zero most frequent value, Appendix A-A1, is summed from the staged copy of x).
//
// X is staged into LDS once per workgroup and gathered from there; one wave per row; the 64 lane totals are combined
// with DPP cross-lane adds.  Two kernels: the stream kernel below, which the library uses, and the expansion kernel
// (an earlier design, kept as a variant that callers can ask for).
#include "cer_device.hpp"

namespace cer {
namespace {

// ------------------------------------------------------------------------------------------------
// batch = 1: the stream kernel
// ------------------------------------------------------------------------------------------------
//
// What bounds a launch of this size on MI355X is the number of vector-memory instructions a compute unit has to
// issue (a wave instruction costs the texture-address unit 16 - 26 clocks whatever its width: 4 lanes per clock), then
// the vector ALU (16 waves share 4 SIMDs) and the LDS gathers.  Hence:
//   * the index stream is read with 16-byte loads: lane l of a window holds PPL consecutive colI positions (8 for
//     16-bit indices), a batch of NW windows is in flight per lane -- 3 loads per 1536 positions instead of 24;
//   * a batch starts at a position that is a multiple of PPL (aligned 16-byte loads); the positions in front of the
//     row's first one belong to a pseudo group of weight 0;
//   * the group structure is turned into per-position weights without any search or data-dependent branch: the lanes
//     that hold a group's end set one bit per boundary in an LDS bitmap of the batch; the index (in the row's list of
//     non-empty groups) of the group a position belongs to is the number of boundary bits in front of it = a prefix
//     count per 32-bit word (one wave scan per batch) + a popcount inside the word; the weight is one LDS read of the
//     list.  None of this depends on the indices or on X, so it runs while the index stream is on its way from HBM;
//   * the stream itself is, per position, an LDS gather of X and one fused multiply-add with the position's weight
//     (a multiply-add costs what an add costs; summing a group first would need the branches this design avoids).

// kNW: windows per batch, 0 = the default (2, 3, 4 for 8-, 16-, 32-bit indices: a batch of 2048, 1536, 1024 positions --
// one batch for the rows of the layer shapes).  Rows of many windows run faster in batches of two windows (the 7-bit
// layer of 7000 indices per row: 15.1 us with 3 windows per batch, 14.2 with 2, 14.9 with 1, 14.7 with 4).
template <typename IdxT, int kNW = 0>
struct GemvShape {
    static constexpr int PPL = 16 / (int)sizeof(IdxT);  // positions per lane and 16-byte load: 16, 8, 4
    static constexpr int WIN = kWave * PPL;             // positions per window (one load per lane)
    static constexpr int NW = kNW ? kNW : (sizeof(IdxT) == 1 ? 2 : (sizeof(IdxT) == 2 ? 3 : 4));  // windows per batch
    static constexpr int BATCH = NW * WIN;              // 2048, 1536, 1024 positions
    static constexpr int NWORDS = BATCH / 32;           // bitmap words per batch: 64, 48, 32 (at most one per lane)
    static constexpr int WPW = WIN / 32;                // bitmap words per window
};

// Inclusive prefix sum over the 64 lanes: four shifted adds inside each row of 16 lanes, then the totals of rows 0
// and 2 are added to rows 1 and 3, then the total of rows 0 - 1 to rows 2 - 3.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
#define CER_SCAN_STEP(CTRL, ROWS) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWS, 0xF, false);
    CER_SCAN_STEP(0x111, 0xF)  // row_shr:1
    CER_SCAN_STEP(0x112, 0xF)  // row_shr:2
    CER_SCAN_STEP(0x114, 0xF)  // row_shr:4
    CER_SCAN_STEP(0x118, 0xF)  // row_shr:8
    CER_SCAN_STEP(0x142, 0xA)  // row_bcast:15 into rows 1 and 3
    CER_SCAN_STEP(0x143, 0xC)  // row_bcast:31 into rows 2 and 3
#undef CER_SCAN_STEP
    return v;
}

// Boundary bitmap of the batch [b0, b0 + BATCH): bit p is set when a list entry ends at position b0 + p + 1, i.e.
// position b0 + p is the last one of its group.  `first` = number of list entries that end at or before b0 (the
// list index of the group position b0 belongs to); `last` = index of the list's second sentinel.  Afterwards
// wpre[j] = first + the number of boundary bits in words 0 .. j-1, and `first` has moved past the batch.
template <typename S>
__device__ __forceinline__ void bitmap_build(const uint32_t* ends, uint32_t last, uint32_t& first, uint32_t b0,
                                             uint32_t* bmp, uint32_t* wpre, uint32_t lane) {
    if (lane < (uint32_t)S::NWORDS) bmp[lane] = 0u;
    wave_lds_sync();
    for (uint32_t i = first;; i += kWave) {
        const uint32_t e = ends[min(i + lane, last)];  // the sentinels (2^32 - 1) are beyond every batch
        const uint32_t rel = e - b0 - 1u;
        if (rel < (uint32_t)S::BATCH) atomicOr(&bmp[rel >> 5], 1u << (rel & 31u));  // LDS operations of a wave run in order
        if (__builtin_amdgcn_readlane(e, kWave - 1) - b0 > (uint32_t)S::BATCH) break;  // wave-uniform
    }
    wave_lds_sync();
    const uint32_t pc = lane < (uint32_t)S::NWORDS ? (uint32_t)__builtin_popcount(bmp[min(lane, (uint32_t)S::NWORDS - 1u)]) : 0u;
    const uint32_t incl = wave_inclusive_scan(pc);
    if (lane < (uint32_t)S::NWORDS) wpre[lane] = first + incl - pc;
    first += __builtin_amdgcn_readlane(incl, kWave - 1);
    wave_lds_sync();
}

// Number of entries of the wave's list (count entries, sentinels behind them) that end at or before position b: the
// list index of the group position b belongs to.
__device__ __forceinline__ uint32_t list_rank_of(const uint32_t* ends, int count, uint32_t b, uint32_t lane) {
    uint32_t f = 0;
    for (int i = 0; i < count; i += kWave) {
        const uint32_t e = ends[min(i + (int)lane, count)];
        f += (uint32_t)__popcll(__ballot(i + (int)lane < count && e <= b));
    }
    return f;
}

// Weights of the PPL positions lane l holds in window W of the batch: wl[k] = value - Omega[0] of the group that
// position b0 + W.WIN + PPL.l + k belongs to (0 in front of the row and behind it).
template <typename S>
__device__ __forceinline__ void window_weights(int W, const uint32_t* bmp, const uint32_t* wpre, const float* wts,
                                               uint32_t lane, float (&wl)[S::PPL]) {
    const uint32_t bit0 = (uint32_t)S::PPL * lane;  // the lane's first bit inside the window
    const uint32_t wj = (uint32_t)W * S::WPW + (bit0 >> 5), sh = bit0 & 31u;
    const uint32_t word = bmp[wj];
    const uint32_t pre = wpre[wj] + (uint32_t)__builtin_popcount(word & ((1u << sh) - 1u));
    const uint32_t field = word >> sh;  // bit k: position k is the last one of its group
    // the LDS address of the position's list entry moves on by one entry behind every boundary bit: one bit-field
    // extract and one shift-add per position
    typedef const float __attribute__((address_space(3))) * LdsFloatPtr;
    uint32_t addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const float*)wts + (pre << 2);
#pragma unroll
    for (int k = 0; k < S::PPL; ++k) {
        wl[k] = *reinterpret_cast<LdsFloatPtr>((uintptr_t)addr);
        if (k + 1 < S::PPL) {
            uint32_t bit;  // written out so that it stays one extract (the compiler turns it into shift + and)
            asm("v_bfe_u32 %0, %1, %2, 1" : "=v"(bit) : "v"(field), "n"(k));
            asm("v_lshl_add_u32 %0, %1, 2, %0" : "+v"(addr) : "v"(bit));  // addr += 4 * bit
        }
    }
}

// Column index of the k-th of the positions packed into one 16-byte load.
template <typename IdxT>
__device__ __forceinline__ uint32_t packed_index(const uint4& q, int k) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if (sizeof(IdxT) == 4) return w[k];
    if (sizeof(IdxT) == 2) return (k & 1) ? (w[k >> 1] >> 16) : (w[k >> 1] & 0xFFFFu);
    return (w[k >> 2] >> (8 * (k & 3))) & 0xFFu;
}

// Appends the non-empty groups among raw groups [j0, tg_end) of the row that starts at group g0 to the wave's list.
// The pointer tiles are requested four at a time (tiles past tg_end read the padding behind the pointer arrays and
// come back empty): a row of 256 raw groups waits for memory once, not four times.
__device__ __forceinline__ int list_append_tiles(const KView& v, bool cser, const float* omega, uint32_t g0, uint32_t j0,
                                                 uint32_t tg_end, uint32_t* ends, float* wts, int count, uint32_t lane) {
    for (; j0 < tg_end; j0 += 4u * kWave) {
        PtrTile p[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) p[t] = load_ptr_tile(v, cser, g0, min(j0 + (uint32_t)t * kWave, tg_end), tg_end, lane);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (j0 + (uint32_t)t * kWave < tg_end)  // wave-uniform
                count = list_append(p[t], omega[p[t].rank < v.K ? p[t].rank : 0u] - v.omega0, ends, wts, count);
    }
    return count;
}

// Byte offset (4 x column index) of the k-th of the positions packed into one 16-byte load: for 8- and 16-bit
// indices one instruction that selects the byte or half-word and shifts it (sub-dword addressing of the vector ALU).
template <typename IdxT>
__device__ __forceinline__ uint32_t packed_offset(const uint4& q, int k, uint32_t two) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t r;
    if (sizeof(IdxT) == 4) {
        r = w[k] << 2;
    } else if (sizeof(IdxT) == 2) {
        const uint32_t d = w[k >> 1];
        if (k & 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(r) : "v"(two), "v"(d));
        else asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(r) : "v"(two), "v"(d));
    } else {
        const uint32_t d = w[k >> 2];
        switch (k & 3) {
            case 0: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(two), "v"(d)); break;
            case 1: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(two), "v"(d)); break;
            case 2: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(two), "v"(d)); break;
            default: asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(two), "v"(d)); break;
        }
    }
    return r;
}

// One batch: gathers and multiply-adds, window by window as the index loads return (they return in order); windows
// that start at or behind the row's end (te) are skipped.
// kLds: X is in LDS at byte address xlds (a literal 0 where the kernel has no static LDS: the gather's address is then
// the shifted index itself); otherwise xsrc points to X in global memory.
template <typename S, typename IdxT, bool kLds>
__device__ __forceinline__ void gemv_batch(const uint4 (&ix)[S::NW], const float* xsrc, uint32_t xlds, uint32_t b0,
                                           uint32_t te, const float (&wl)[S::NW][S::PPL],
                                           float& acc0, float& acc1) {
#pragma unroll
    for (int W = 0; W < S::NW; ++W) {
        if (W > 0 && b0 + (uint32_t)W * S::WIN >= te) break;  // wave-uniform
        float xv[S::PPL];
        if (kLds) {  // X in LDS: 32-bit byte addresses
            typedef const float __attribute__((address_space(3))) * LdsFloatPtr;
            uint32_t two = 2u;
            asm("" : "+v"(two));  // the shift count in a vector register (sub-dword forms take no constants)
#pragma unroll
            for (int k = 0; k < S::PPL; ++k)
                xv[k] = *reinterpret_cast<LdsFloatPtr>((uintptr_t)(xlds + packed_offset<IdxT>(ix[W], k, two)));
        } else {
#pragma unroll
            for (int k = 0; k < S::PPL; ++k) xv[k] = xsrc[packed_index<IdxT>(ix[W], k)];
        }
#pragma unroll
        for (int k = 0; k < S::PPL; k += 2) {
            acc0 = fmaf(xv[k], wl[W][k], acc0);
            acc1 = fmaf(xv[k + 1], wl[W][k + 1], acc1);
        }
    }
}

// kOneRow: the launch gives every wave at most one row (matrices of up to 16 rows per compute unit and workgroup
// slot), so the loop over a wave's rows and what it keeps alive fall away.  Such a launch may also give a row to
// 2, 4 or 8 consecutive waves of a workgroup (matrices of so few rows that one wave per row would leave most of the
// chip idle): the row's windows of WIN positions are dealt to them in equal contiguous shares, every wave builds the
// row's group list and starts its bitmap at its own share, and the partial sums meet in LDS (added in wave order by
// the first of them).  `rows_and_parts` = rows per workgroup | log2(waves per row) << 28.
template <typename IdxT, bool kXinLds, bool kVec4, bool kCser, bool kOneRow>
__global__ __launch_bounds__(1024) void cer_gemv_kernel(const void* __restrict__ colI_, const uint2* __restrict__ rowInfo_,
                                                        const float* __restrict__ X, float* __restrict__ Y,
                                                        const uint32_t* __restrict__ omegaPtr_, const float* __restrict__ omega_,
                                                        uint32_t n_, uint32_t m_, uint32_t K_, uint32_t rows_and_parts,
                                                        uint32_t gcap, float omega0_, const void* __restrict__ omegaI_,
                                                        const float* __restrict__ T, int omegaI_bits_, int omega_in_lds) {
    // Plain pointers and integers, the ones the first instructions need in front: the first 16 dwords of a kernel's
    // arguments are preloaded into scalar registers when the wave is launched (the library is built with kernel-
    // argument preloading), so the row descriptor and the first X loads do not wait for a load of the arguments.
    using S = GemvShape<IdxT>;
    KView v;
    v.colI = colI_; v.omegaPtr = omegaPtr_; v.rowPtr = nullptr; v.rowInfo = rowInfo_; v.omegaI = omegaI_; v.omega = omega_;
    v.K = K_; v.omegaI_bits = omegaI_bits_; v.cser = kCser ? 1 : 0; v.m = m_; v.n = n_; v.omega0 = omega0_;
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t nwaves = blockDim.x >> 6;

    // LDS: [X: n floats, rounded to 4] [Omega: K floats, optional] [ends | wts: nwaves x (gcap + 3)]
    //      [bitmap | word prefix: nwaves x NWORDS]
    float* xs = reinterpret_cast<float*>(smem);
    const uint32_t x_floats = kXinLds ? ((v.n + 3u) & ~3u) : 0u;
    float* oms = xs + x_floats;
    const uint32_t om_floats = omega_in_lds ? ((v.K + 3u) & ~3u) : 0u;
    const uint32_t lcap = gcap + 3u;  // the pseudo group in front of the row, the groups, two sentinels
    uint32_t* list0 = reinterpret_cast<uint32_t*>(oms + om_floats);
    uint32_t* ends = list0 + wave * lcap;
    float* wts = reinterpret_cast<float*>(list0 + nwaves * lcap) + wave * lcap;
    uint32_t* bmp = list0 + 2u * nwaves * lcap + wave * (uint32_t)S::NWORDS;
    uint32_t* wpre = list0 + 2u * nwaves * lcap + (nwaves + wave) * (uint32_t)S::NWORDS;
    const float* omega = omega_in_lds ? oms : v.omega;
    const float* xsrc = kXinLds ? xs : X;
    const uint32_t xlds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)xs;  // LDS byte address of X

    const uint32_t rows_per_block = rows_and_parts & 0x0FFFFFFFu;
    const uint32_t part_shift = kOneRow ? rows_and_parts >> 28 : 0u;
    const uint32_t parts = 1u << part_shift, part = wave & (parts - 1u);
    const uint32_t row_begin = blockIdx.x * rows_per_block;
    const uint32_t row_end = min(v.m, row_begin + rows_per_block);
    const IdxT* colI = static_cast<const IdxT*>(v.colI);
    uint32_t r = row_begin + (wave >> part_shift);  // wave-uniform: the descriptor loads below are scalar loads

    // (1) descriptor of the wave's first row: {first group, first colI offset} of rows r and r+1
    uint32_t g0 = 0, g1 = 0, rs = 0, re = 0;
    if (r < row_end) {
        const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];
        g0 = d0.x; rs = d0.y; g1 = d1.x; re = d1.y;
    }

    // (2) X and Omega on their way to LDS: up to eight 16-byte loads per thread, only those that hold part of X
    //     (wave-uniform tests), in named registers (an indexed array would end up in scratch memory)
    typedef float F4 __attribute__((ext_vector_type(4)));
    F4 xr0, xr1, xr2, xr3, xr4, xr5, xr6, xr7;  // a register is stored only where it was loaded (the same bound)
    const uint32_t n4 = kVec4 ? (v.n >> 2) : 0u;
    const F4* X4 = reinterpret_cast<const F4*>(X);
    const uint32_t wave_first = wave * kWave;  // the wave's first thread
#define CER_STAGE_IDX(k) ((k) * blockDim.x + threadIdx.x)
#define CER_STAGE_LOAD(k) if ((k) * blockDim.x + wave_first < n4) xr##k = X4[min(CER_STAGE_IDX(k), n4 - 1u)]
    if (kXinLds && kVec4) {
        CER_STAGE_LOAD(0); CER_STAGE_LOAD(1); CER_STAGE_LOAD(2); CER_STAGE_LOAD(3);
        CER_STAGE_LOAD(4); CER_STAGE_LOAD(5); CER_STAGE_LOAD(6); CER_STAGE_LOAD(7);
    }
    const float om_l = v.omega[lane < v.K ? lane : 0u];  // Omega[lane]: lets a wave look values up by lane shuffle
    __builtin_amdgcn_sched_barrier(0);
    // The waves do not meet at a barrier once X is staged (that would make every wave wait for the slowest one's group
    // list and weights): each wave counts itself in when its part of X is in LDS and, before its first gather, waits
    // until all have.  The counter starts at zero: one early barrier, which every wave reaches before it waits for
    // anything (and which keeps the X loads of the whole workgroup ahead of the first index load in the memory pipe).
    __shared__ uint32_t s_staged;
    if (kXinLds || omega_in_lds) {
        if (threadIdx.x == 0) s_staged = 0u;
        __syncthreads();
    }
    __builtin_amdgcn_sched_barrier(0);

    // (3) first row: its first 64 group pointers and the indices of its first batch, all unconditional.  A batch
    //     starts at a multiple of PPL positions; what lies in front of the row gets the weight 0.
    const PtrTile pt0 = load_ptr_tile_first(v, kCser, g0, g0, min(g1, g0 + min(gcap, (uint32_t)kWave)), lane);
    uint4 idx0[S::NW];  // used by one piece of code only (no merge with re-loaded values, which would make the
                        // compiler wait for all of them at the merge point)
    uint32_t b00 = rs & ~((uint32_t)S::PPL - 1u);
    uint32_t re0 = re;  // end of this wave's share of the first row
    if (kOneRow && parts > 1u) {
        const uint32_t nwin = (re - b00 + (uint32_t)S::WIN - 1u) / (uint32_t)S::WIN;
        const uint32_t share = ((nwin + parts - 1u) >> part_shift) * (uint32_t)S::WIN;
        const uint32_t mine = b00 + part * share;
        if (mine < re) { b00 = mine; re0 = min(re, mine + share); } else { re0 = b00; }  // an empty share does nothing
    }
    {
        // a window that lies behind the row's end asks for the first window again: the loads stay unconditional,
        // but the next rows' indices are not fetched from memory a second time
        const uint4* p = reinterpret_cast<const uint4*>(colI + b00) + lane;
#pragma unroll
        for (int W = 0; W < S::NW; ++W) idx0[W] = p[(b00 + (uint32_t)W * S::WIN < re0 ? W : 0) * kWave];
    }
    // a first row of more than 64 raw groups: the next three pointer tiles as well (behind the indices in the queue)
    const uint32_t tg_end0 = min(g1, g0 + gcap);
    const bool many0 = tg_end0 - g0 > (uint32_t)kWave;  // wave-uniform
    PtrTile pt1, pt2, pt3;
    if (many0) {
        pt1 = load_ptr_tile(v, kCser, g0, min(g0 + 1u * kWave, tg_end0), tg_end0, lane);
        pt2 = load_ptr_tile(v, kCser, g0, min(g0 + 2u * kWave, tg_end0), tg_end0, lane);
        pt3 = load_ptr_tile(v, kCser, g0, min(g0 + 3u * kWave, tg_end0), tg_end0, lane);
    }
    __builtin_amdgcn_sched_barrier(0);

    // (4) finish staging.  Appendix A-A1 needs sum_i X[i] when the most frequent value is not 0: every thread adds
    //     up what it stages (a short chain), the wave's total goes to LDS before the wave counts itself in.
    __shared__ float s_xsum[16];
    const bool want_xsum = kXinLds && v.omega0 != 0.f;  // uniform over the grid
    float xpart = 0.f;
    if (kXinLds) {
        if (kVec4) {
            F4* xs4 = reinterpret_cast<F4*>(xs);
#define CER_STAGE_STORE(k) if (CER_STAGE_IDX(k) < n4) xs4[CER_STAGE_IDX(k)] = xr##k
            CER_STAGE_STORE(0); CER_STAGE_STORE(1); CER_STAGE_STORE(2); CER_STAGE_STORE(3);
            CER_STAGE_STORE(4); CER_STAGE_STORE(5); CER_STAGE_STORE(6); CER_STAGE_STORE(7);
#define CER_STAGE_SUM(k) if (CER_STAGE_IDX(k) < n4) xpart += (xr##k.x + xr##k.y) + (xr##k.z + xr##k.w)
            if (want_xsum) {
                CER_STAGE_SUM(0); CER_STAGE_SUM(1); CER_STAGE_SUM(2); CER_STAGE_SUM(3);
                CER_STAGE_SUM(4); CER_STAGE_SUM(5); CER_STAGE_SUM(6); CER_STAGE_SUM(7);
            }
#undef CER_STAGE_SUM
            for (uint32_t i = 8u * blockDim.x + threadIdx.x; i < n4; i += blockDim.x) {
                const F4 x4 = X4[i];
                xs4[i] = x4;
                xpart += (x4.x + x4.y) + (x4.z + x4.w);
            }
        }
        for (uint32_t i = (n4 << 2) + threadIdx.x; i < v.n; i += blockDim.x) {
            const float x1 = X[i];
            xs[i] = x1;
            xpart += x1;
        }
        if (want_xsum) {
            xpart = wave_sum(xpart);
            if (lane == 0) s_xsum[wave] = xpart;
        }
    }
#undef CER_STAGE_STORE
#undef CER_STAGE_LOAD
#undef CER_STAGE_IDX
    if (omega_in_lds) {
        if (threadIdx.x < min(v.K, (uint32_t)kWave)) oms[threadIdx.x] = om_l;  // the first wave
        for (uint32_t i = kWave + threadIdx.x; i < v.K; i += blockDim.x) oms[i] = v.omega[i];
    }
    if (kXinLds || omega_in_lds) {
        wave_lds_sync();  // the LDS operations of a wave are executed in order: its stores, then its count
        if (lane == 0) __hip_atomic_fetch_add(&s_staged, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    // With at most 64 values and at most 64 raw groups in the first row, its group list, the first batch's bitmap and
    // the weights of the first batch are built here, before the workgroup barrier, from the pointer tile (which
    // arrives ahead of the indices) and a lane shuffle of Omega.
    int count0 = -1;   // entries of the first row's list, the pseudo group included; -1: not built here
    uint32_t first = 0;  // list index of the group the next batch's first position belongs to
    float wl0[S::NW][S::PPL];
    if (v.K <= (uint32_t)kWave && g1 - g0 <= min(gcap, (uint32_t)kWave)) {
        const float w = __shfl(om_l, (int)(pt0.rank & 63u), kWave) - v.omega0;
        if (lane == 0) { ends[0] = rs; wts[0] = 0.f; }
        count0 = list_append(pt0, w, ends, wts, 1);
        list_close(ends, wts, count0, lane);
        if (count0 > 1) {
            wave_lds_sync();
            first = (kOneRow && part > 0u) ? list_rank_of(ends, count0, b00, lane) : (rs > b00 ? 0u : 1u);
            bitmap_build<S>(ends, (uint32_t)count0 + 1u, first, b00, bmp, wpre, lane);
#pragma unroll
            for (int W = 0; W < S::NW; ++W)
                if (W == 0 || b00 + (uint32_t)W * S::WIN < re0) window_weights<S>(W, bmp, wpre, wts, lane, wl0[W]);
        }
    }
    if (kXinLds || omega_in_lds) {
        // every wave of the workgroup has counted itself in, or will without waiting for anything but its own loads;
        // the bound on the spin only keeps a broken launch from hanging
        for (uint32_t spin = 0; spin < (1u << 22); ++spin) {
            if (__hip_atomic_load(&s_staged, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= nwaves) break;
            __builtin_amdgcn_s_sleep(1);
        }
        wave_lds_sync();
    }

    // Appendix A-A1: Omega[0] . sum_i X[i].  With X staged in LDS the waves' totals are in LDS by now (added in wave
    // order); otherwise the launcher has computed the sum into T.
    float t_off = 0.f;
    if (v.omega0 != 0.f) {  // uniform over the grid
        float tsum;
        if (kXinLds) {
            tsum = 0.f;
            for (uint32_t w = 0; w < nwaves; ++w) tsum += s_xsum[w];
        } else {
            tsum = T[0];
        }
        t_off = v.omega0 * tsum;
    }

    // The first batch of the first row runs from the prefetched indices when its list is ready (the common case);
    // everything else -- later batches, rows with many groups, later rows -- goes through the general loop below.
    float acc0 = 0.f, acc1 = 0.f;
    bool resume = false;
    uint32_t te0 = re0;  // end of the first row's first tile of groups (of this wave's share of it)
    if (count0 < 0 && r < row_end && g1 > g0) {
        // more than 64 values or raw groups: the list of the first tile is built here, with Omega from LDS; the
        // indices of its first batch are the ones requested in the prologue
        if (tg_end0 != g1) te0 = uniform(v.omegaPtr[tg_end0]);
        if (lane == 0) { ends[0] = rs; wts[0] = 0.f; }
        count0 = list_append(pt0, omega[pt0.rank < v.K ? pt0.rank : 0u] - v.omega0, ends, wts, 1);
        if (many0) {
            count0 = list_append(pt1, omega[pt1.rank < v.K ? pt1.rank : 0u] - v.omega0, ends, wts, count0);
            count0 = list_append(pt2, omega[pt2.rank < v.K ? pt2.rank : 0u] - v.omega0, ends, wts, count0);
            count0 = list_append(pt3, omega[pt3.rank < v.K ? pt3.rank : 0u] - v.omega0, ends, wts, count0);
            count0 = list_append_tiles(v, kCser, omega, g0, g0 + 4u * kWave, tg_end0, ends, wts, count0, lane);
        }
        list_close(ends, wts, count0, lane);
        if (count0 > 1) {
            wave_lds_sync();
            first = (kOneRow && part > 0u) ? list_rank_of(ends, count0, b00, lane) : (rs > b00 ? 0u : 1u);
            bitmap_build<S>(ends, (uint32_t)count0 + 1u, first, b00, bmp, wpre, lane);
#pragma unroll
            for (int W = 0; W < S::NW; ++W)
                if (W == 0 || b00 + (uint32_t)W * S::WIN < te0) window_weights<S>(W, bmp, wpre, wts, lane, wl0[W]);
        }
    }
    if (r < row_end && count0 > 1 && b00 < te0) {
        gemv_batch<S, IdxT, kXinLds>(idx0, xsrc, xlds, b00, te0, wl0, acc0, acc1);
        resume = true;
    }

    bool first_row = true;
    float y_share = 0.f;
    for (; r < row_end; r += nwaves) {
        if (!first_row) {
            const uint2 e0 = v.rowInfo[r], e1 = v.rowInfo[r + 1];
            g0 = e0.x; rs = e0.y; g1 = e1.x; re = e1.y;
            acc0 = acc1 = 0.f;
        }
        // a row is one tile unless it has more raw groups than the wave's list holds
        for (uint32_t tg = g0; tg < g1; tg += gcap) {
            const uint32_t tg_end = min(g1, tg + gcap);
            const uint32_t ts = tg == g0 ? rs : uniform(v.omegaPtr[tg]);
            uint32_t te = tg_end == g1 ? re : uniform(v.omegaPtr[tg_end]);
            const bool resumed = first_row && resume && tg == g0;  // the tile's first batch is done, its list is live
            uint32_t b0 = ts & ~((uint32_t)S::PPL - 1u);
            if (kOneRow && parts > 1u) { b0 = b00; te = te0; }  // a shared row is one tile of groups: this wave's share
            int count;
            if (resumed) {
                count = count0;
                b0 += S::BATCH;
            } else {
                const bool pre = first_row && tg == g0;
                if (pre && count0 >= 0) {
                    count = count0;
                } else {
                    // the pseudo group in front of the tile, then its non-empty groups
                    if (lane == 0) { ends[0] = ts; wts[0] = 0.f; }
                    count = list_append_tiles(v, kCser, omega, g0, tg, tg_end, ends, wts, 1, lane);
                    list_close(ends, wts, count, lane);
                }
                wave_lds_sync();
                first = ts > b0 ? 0u : 1u;
            }
            if (count > 1 && b0 < te) {
                // Two sets of index registers: the next batch is requested before the current one is summed, so
                // that a wave working alone on a long row (the others of its compute unit are done) does not
                // wait out the memory latency once per batch.  Past the row's end the current batch is requested
                // again (in bounds, unused) to keep the loads unconditional.
                uint4 ixa[S::NW], ixb[S::NW];
                float wl[S::NW][S::PPL];
#define CER_REQUEST(ix, b)                                                                       \
    {                                                                                            \
        const uint4* p_ = reinterpret_cast<const uint4*>(colI + (b)) + lane;                     \
        _Pragma("unroll") for (int W = 0; W < S::NW; ++W)                                        \
            ix[W] = p_[((b) + (uint32_t)W * S::WIN < te ? W : 0) * kWave];                        \
    }
#define CER_BATCH(ix, b)                                                                         \
    bitmap_build<S>(ends, (uint32_t)count + 1u, first, b, bmp, wpre, lane);                      \
    _Pragma("unroll") for (int W = 0; W < S::NW; ++W)                                            \
        if (W == 0 || (b) + (uint32_t)W * S::WIN < te) window_weights<S>(W, bmp, wpre, wts, lane, wl[W]); \
    gemv_batch<S, IdxT, kXinLds>(ix, xsrc, xlds, b, te, wl, acc0, acc1);
                CER_REQUEST(ixa, b0)
                for (;;) {
                    const uint32_t b1 = b0 + S::BATCH;
                    CER_REQUEST(ixb, b1 < te ? b1 : b0)
                    CER_BATCH(ixa, b0)
                    if (b1 >= te) break;
                    const uint32_t b2 = b1 + S::BATCH;
                    CER_REQUEST(ixa, b2 < te ? b2 : b1)
                    CER_BATCH(ixb, b1)
                    if (b2 >= te) break;
                    b0 = b2;
                }
#undef CER_BATCH
#undef CER_REQUEST
            }
            wave_lds_sync();  // the list is rebuilt by the next tile / row
        }
        const float y = wave_sum(acc0 + acc1);
        if (kOneRow && parts > 1u) { y_share = y; break; }
        if (lane == 0) Y[r] = y + t_off;
        if (kOneRow) break;
        first_row = false;
    }
    if (kOneRow && parts > 1u) {  // uniform over the workgroup
        __shared__ float s_share[16];
        if (lane == 0) s_share[wave] = y_share;
        __syncthreads();
        if (part == 0u && r < row_end && lane == 0) {
            float y = s_share[wave];
            for (uint32_t q = 1; q < parts; ++q) y += s_share[wave + q];
            Y[r] = y + t_off;
        }
    }
}


// ------------------------------------------------------------------------------------------------
// batch = 1: the stream kernel over the rank table (codebooks of at most 256 values, X in LDS)
// ------------------------------------------------------------------------------------------------
//
// What a launch of a few microseconds spends most of its time on is waiting for memory that has to be asked for in
// sequence: the row descriptor, then the group pointers and the first indices it locates, each a full trip to HBM.
// For codebooks of at most 256 values the handle carries a rank table (derived from the format arrays, one record of
// Kp = 4 .. 256 32-bit words per row at a fixed stride): word 0 is the row's first colI position, word k the end of its
// group of rank k (the previous word where the row has no element of that rank).  A wave finds its record from the row
// number alone, so the first trip to memory already brings the row's start, its end and every group boundary; the
// second trip fetches the indices, and the group list, the boundary bitmap and the weights of the first batch are
// built while it is on its way.  CER and CSER handles have the same table, so the kernel does not know the format.
// Everything else -- batches, windows, bitmap, shared rows, the staging of X -- is as in the kernel above.
// kBigX: every wave of the workgroup has six whole 16-byte loads of X (6 x the workgroup size x 16 bytes <= 4n).
// kShortBatch: batches of two windows (16-bit indices, rows of more than three windows on average).
template <typename IdxT, bool kVec4, bool kOneRow, bool kBigX, bool kShortBatch = false>
__global__ __launch_bounds__(1024) void cer_gemv_tab_kernel(const uint32_t* __restrict__ tab, const float* __restrict__ X,
                                                            const float* __restrict__ omega_, const void* __restrict__ colI_,
                                                            float* __restrict__ Y, uint32_t n, uint32_t m,
                                                            uint32_t rows_per_block, uint32_t meta) {
    // 14 dwords of arguments: all of them are preloaded into scalar registers when a wave starts (the library is
    // built with kernel-argument preloading), so no instruction in front of the first memory request waits for a
    // load of the argument block.  For the same reason the workgroup size comes from `meta`, not from the dispatch
    // packet, and Omega[0] from Omega.  meta = K | log2(words per record) << 9 | log2(waves per row) << 13 |
    // waves per workgroup << 16.
    using S = GemvShape<IdxT, (kShortBatch && sizeof(IdxT) == 2) ? 2 : 0>;
    extern __shared__ __align__(16) unsigned char smem[];
    const uint32_t K = meta & 0x1FFu, tab_shift = (meta >> 9) & 0xFu;
    const uint32_t nwaves = meta >> 16, bdim = nwaves * kWave;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);

    // LDS: [X: n floats, rounded to 4] [ends | wts: nwaves x lcap] [bitmap | word prefix: nwaves x NWORDS]
    //      [counter of staged waves, 16 sums of X, 16 partial row sums].  The kernel has no static LDS, so X sits at
    //      LDS address 0 and a gather's address is 4 x the column index.
    float* xs = reinterpret_cast<float*>(smem);
    const uint32_t x_floats = (n + 3u) & ~3u;
    const uint32_t last_word = (1u << tab_shift) - 1u;
    const uint32_t ntiles = (last_word >> 6) + 1u;  // 64 ranks per tile: 1, 2 or 4 tiles
    const uint32_t lcap = max(last_word, 63u) + 5u;  // the pseudo group in front of the row, the groups, two sentinels
    uint32_t* list0 = reinterpret_cast<uint32_t*>(xs + x_floats);
    uint32_t* ends = list0 + wave * lcap;
    float* wts = reinterpret_cast<float*>(list0 + nwaves * lcap) + wave * lcap;
    uint32_t* bmp = list0 + 2u * nwaves * lcap + wave * (uint32_t)S::NWORDS;
    uint32_t* wpre = list0 + 2u * nwaves * lcap + (nwaves + wave) * (uint32_t)S::NWORDS;
    uint32_t* s_staged = list0 + 2u * nwaves * lcap + 2u * nwaves * (uint32_t)S::NWORDS;
    float* s_xsum = reinterpret_cast<float*>(s_staged + 4);
    float* s_share = s_xsum + 16;

    const uint32_t part_shift = kOneRow ? (meta >> 13) & 0x7u : 0u;
    const uint32_t parts = 1u << part_shift, part = wave & (parts - 1u);
    const uint32_t row_begin = blockIdx.x * rows_per_block;
    const uint32_t row_end = min(m, row_begin + rows_per_block);
    const IdxT* colI = static_cast<const IdxT*>(colI_);
    uint32_t r = row_begin + (wave >> part_shift);  // wave-uniform

    // (1) the row's record, one word per lane and tile (a wave without a row reads the last row's and ignores it),
    //     and Omega: Omega[lane] (lane 0: Omega[0]; the next lane's value is the one of the group of rank lane + 1),
    //     for further tiles the value of the lane's rank itself
    auto load_rec = [&](uint32_t row, uint32_t t) { return tab[((size_t)row << tab_shift) + min(t * kWave + lane, last_word)]; };
    uint32_t rec = load_rec(min(r, m - 1u), 0u), rec1 = 0u, rec2 = 0u, rec3 = 0u;
    const float om_l = omega_[min(lane, K - 1u)];
    float wq0 = 0.f, wq1 = 0.f, wq2 = 0.f, wq3 = 0.f;
    if (ntiles > 1u) {  // wave-uniform
        rec1 = load_rec(min(r, m - 1u), 1u);
        wq0 = omega_[min(lane + 1u, K - 1u)];  // lane 63: rank 64, which the shifted Omega[lane] cannot supply
        wq1 = omega_[min(1u * kWave + lane + 1u, K - 1u)];
    }
    if (ntiles > 2u) {
        rec2 = load_rec(min(r, m - 1u), 2u);
        rec3 = load_rec(min(r, m - 1u), 3u);
        wq2 = omega_[min(2u * kWave + lane + 1u, K - 1u)];
        wq3 = omega_[min(3u * kWave + lane + 1u, K - 1u)];
    }
    __builtin_amdgcn_sched_barrier(0);
    // The counter of staged waves starts at zero: one early barrier that no wave waits at for memory -- in front of
    // the X loads, whose issue is what takes time (a compute unit's vector-memory pipeline accepts a 16-byte-per-lane
    // load about every 26 clocks: 128 of them for 98 KB of X).
    if (threadIdx.x == 0) *s_staged = 0u;
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);

    // (2) X on its way to LDS: up to eight 16-byte loads per thread, only those that hold part of X (wave-uniform
    //     tests), all in front of the index loads (the earlier X is requested the earlier it is staged: measured
    //     with 0 .. 8 loads in front).  When X is large enough for every wave to have six whole loads (what takes
    //     time to stage), these are unconditional: the compiler can then wait for the record alone -- after
    //     conditionally issued loads it has to assume that none was issued, and waits for all of them.
    typedef float F4 __attribute__((ext_vector_type(4)));
    F4 xr0, xr1, xr2, xr3, xr4, xr5, xr6, xr7;
    const uint32_t n4 = kVec4 ? (n >> 2) : 0u;
    const F4* X4 = reinterpret_cast<const F4*>(X);
    F4* xs4 = reinterpret_cast<F4*>(xs);
    const uint32_t wave_first = wave * kWave;
    constexpr bool big = kVec4 && kBigX;
#define CER_STAGE_IDX(k) ((k) * bdim + threadIdx.x)
#define CER_STAGE_LOAD(k) if ((k) * bdim + wave_first < n4) xr##k = X4[min(CER_STAGE_IDX(k), n4 - 1u)]
#define CER_STAGE_STORE(k) if (CER_STAGE_IDX(k) < n4) xs4[CER_STAGE_IDX(k)] = xr##k
#define CER_STAGE_SUM(k) if (CER_STAGE_IDX(k) < n4) xpart += (xr##k.x + xr##k.y) + (xr##k.z + xr##k.w)
    uint32_t rs, re;
    float omega0, w_l;  // Omega[0] and the weight of the group of rank lane + 1 (ranks stay below K <= 64)
#define CER_RECORD_HERE                                                                                       \
    if (r >= row_end) rec = rec1 = rec2 = rec3 = 0u; /* no row: no groups */                                  \
    rs = (uint32_t)__builtin_amdgcn_readlane((int)rec, 0);                                                    \
    re = ntiles == 1u ? (uint32_t)__builtin_amdgcn_readlane((int)rec, (int)(last_word & 63u))                 \
                      : (uint32_t)__builtin_amdgcn_readlane((int)(ntiles == 2u ? rec1 : rec3), 63);           \
    omega0 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(om_l)));                            \
    w_l = (ntiles > 1u ? wq0 : __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(om_l), 0x130 /* wave_shl:1 */, 0xF, 0xF, false))) - omega0;
    if (big) {
        xr0 = X4[CER_STAGE_IDX(0)]; xr1 = X4[CER_STAGE_IDX(1)]; xr2 = X4[CER_STAGE_IDX(2)];
        xr3 = X4[CER_STAGE_IDX(3)]; xr4 = X4[CER_STAGE_IDX(4)]; xr5 = X4[CER_STAGE_IDX(5)];
        CER_STAGE_LOAD(6); CER_STAGE_LOAD(7);
        __builtin_amdgcn_sched_barrier(0);
        CER_RECORD_HERE
    } else {
        if (kVec4) {
            CER_STAGE_LOAD(0); CER_STAGE_LOAD(1); CER_STAGE_LOAD(2); CER_STAGE_LOAD(3);
            CER_STAGE_LOAD(4); CER_STAGE_LOAD(5); CER_STAGE_LOAD(6); CER_STAGE_LOAD(7);
        }
        __builtin_amdgcn_sched_barrier(0);
        CER_RECORD_HERE
    }
#undef CER_RECORD_HERE
    __builtin_amdgcn_sched_barrier(0);

    // (3) the record is here (and with it Omega): the row's extent, this wave's share of it, the indices of its
    //     first batch
    uint32_t b00 = rs & ~((uint32_t)S::PPL - 1u);
    uint32_t re0 = re;
    if (kOneRow && parts > 1u) {
        const uint32_t nwin = (re - b00 + (uint32_t)S::WIN - 1u) / (uint32_t)S::WIN;
        const uint32_t share = ((nwin + parts - 1u) >> part_shift) * (uint32_t)S::WIN;
        const uint32_t mine = b00 + part * share;
        if (mine < re) { b00 = mine; re0 = min(re, mine + share); } else { re0 = b00; }
    }
    __builtin_amdgcn_sched_barrier(0);
    uint4 idx0[S::NW];
    {
        // a window that lies behind the row's end asks for the first window again: the loads stay unconditional,
        // but the next rows' indices are not fetched from memory a second time
        const uint4* p = reinterpret_cast<const uint4*>(colI + b00) + lane;
#pragma unroll
        for (int W = 0; W < S::NW; ++W) idx0[W] = p[(b00 + (uint32_t)W * S::WIN < re0 ? W : 0) * kWave];
    }
    __builtin_amdgcn_sched_barrier(0);

    // (4) X goes to LDS (only the index loads are behind it in the queue) and the wave counts itself in; Appendix
    //     A-A1: every thread adds up what it stages, the wave's total goes to LDS before the count
    const bool want_xsum = omega0 != 0.f;  // uniform over the grid
    float xpart = 0.f;
    if (kVec4) {
        CER_STAGE_STORE(0); CER_STAGE_STORE(1); CER_STAGE_STORE(2); CER_STAGE_STORE(3);
        CER_STAGE_STORE(4); CER_STAGE_STORE(5); CER_STAGE_STORE(6); CER_STAGE_STORE(7);
        if (want_xsum) {
            CER_STAGE_SUM(0); CER_STAGE_SUM(1); CER_STAGE_SUM(2); CER_STAGE_SUM(3);
            CER_STAGE_SUM(4); CER_STAGE_SUM(5); CER_STAGE_SUM(6); CER_STAGE_SUM(7);
        }
#undef CER_STAGE_SUM
#undef CER_STAGE_STORE
        for (uint32_t i = 8u * bdim + threadIdx.x; i < n4; i += bdim) {
            const F4 x4 = X4[i];
            xs4[i] = x4;
            xpart += (x4.x + x4.y) + (x4.z + x4.w);
        }
    }
#undef CER_STAGE_LOAD
#undef CER_STAGE_IDX
    for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += bdim) {
        const float x1 = X[i];
        xs[i] = x1;
        xpart += x1;
    }
    if (want_xsum) {
        xpart = wave_sum(xpart);
        if (lane == 0) s_xsum[wave] = xpart;
    }
    wave_lds_sync();  // the LDS operations of a wave are executed in order: its stores, then its count
    if (lane == 0) __hip_atomic_fetch_add(s_staged, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __builtin_amdgcn_sched_barrier(0);

    // (5) group list, bitmap and weights of the first batch, while the indices are on their way: lane l holds the
    //     group of rank l + 1, which ends where the next lane's group begins
    // tile t of a record: lane l holds the group of rank 64 t + l + 1; `next` = the first word of the next tile
    auto record_tile = [&](uint32_t rc, uint32_t next, uint32_t t) {
        PtrTile p;
        p.s = rc;
        p.e = (uint32_t)__builtin_amdgcn_update_dpp((int)rc, (int)rc, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
        if (lane == (uint32_t)kWave - 1u) p.e = next;
        if (t * kWave + lane >= last_word) p.e = p.s;
        p.rank = t * kWave + lane + 1u;
        return p;
    };
    // the row's list from its record: the pseudo group in front of the row, then the non-empty groups
    auto build_list = [&]() {
        if (lane == 0) { ends[0] = rs; wts[0] = 0.f; }
        const uint32_t n1 = (uint32_t)__builtin_amdgcn_readlane((int)rec1, 0);
        int count = list_append(record_tile(rec, n1, 0u), w_l, ends, wts, 1);
        if (ntiles > 1u) {
            const uint32_t n2 = (uint32_t)__builtin_amdgcn_readlane((int)rec2, 0);
            count = list_append(record_tile(rec1, n2, 1u), wq1 - omega0, ends, wts, count);
        }
        if (ntiles > 2u) {
            const uint32_t n3 = (uint32_t)__builtin_amdgcn_readlane((int)rec3, 0);
            count = list_append(record_tile(rec2, n3, 2u), wq2 - omega0, ends, wts, count);
            count = list_append(record_tile(rec3, 0u, 3u), wq3 - omega0, ends, wts, count);
        }
        list_close(ends, wts, count, lane);
        return count;
    };
    int count0 = build_list();
    uint32_t first = 0;
    float wl0[S::NW][S::PPL];
    const bool run0 = count0 > 1 && b00 < re0;  // wave-uniform
    if (run0) {
        wave_lds_sync();
        first = (kOneRow && part > 0u) ? list_rank_of(ends, count0, b00, lane) : (rs > b00 ? 0u : 1u);
        bitmap_build<S>(ends, (uint32_t)count0 + 1u, first, b00, bmp, wpre, lane);
#pragma unroll
        for (int W = 0; W < S::NW; ++W)
            if (W == 0 || b00 + (uint32_t)W * S::WIN < re0) window_weights<S>(W, bmp, wpre, wts, lane, wl0[W]);
    }
    __builtin_amdgcn_sched_barrier(0);

    // every wave of the workgroup counts itself in without waiting for anything but its own loads; the bound on the
    // spin only keeps a broken launch from hanging
    for (uint32_t spin = 0; spin < (1u << 22); ++spin) {
        if (__hip_atomic_load(s_staged, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= nwaves) break;
        __builtin_amdgcn_s_sleep(1);
    }
    wave_lds_sync();
    float t_off = 0.f;
    if (want_xsum) {
        float tsum = 0.f;
        for (uint32_t w = 0; w < nwaves; ++w) tsum += s_xsum[w];
        t_off = omega0 * tsum;
    }

    // (6) the stream: the first batch from the prefetched indices, then the rest of the row, then further rows
    float acc0 = 0.f, acc1 = 0.f;
    if (run0) gemv_batch<S, IdxT, true>(idx0, xs, 0u, b00, re0, wl0, acc0, acc1);
    bool first_row = true;
    float y_share = 0.f;
    for (; r < row_end; r += nwaves) {
        uint32_t b0, te;
        int count;
        if (first_row) {
            count = run0 ? count0 : 0;
            b0 = b00 + (uint32_t)S::BATCH;
            te = re0;
        } else {
            rec = load_rec(r, 0u);
            if (ntiles > 1u) rec1 = load_rec(r, 1u);
            if (ntiles > 2u) { rec2 = load_rec(r, 2u); rec3 = load_rec(r, 3u); }
            rs = (uint32_t)__builtin_amdgcn_readlane((int)rec, 0);
            re = ntiles == 1u ? (uint32_t)__builtin_amdgcn_readlane((int)rec, (int)(last_word & 63u))
                              : (uint32_t)__builtin_amdgcn_readlane((int)(ntiles == 2u ? rec1 : rec3), 63);
            acc0 = acc1 = 0.f;
            count = build_list();
            wave_lds_sync();
            b0 = rs & ~((uint32_t)S::PPL - 1u);
            te = re;
            first = rs > b0 ? 0u : 1u;
        }
        if (count > 1 && b0 < te) {
            // two sets of index registers: the next batch is requested before the current one is summed
            uint4 ixa[S::NW], ixb[S::NW];
            float wl[S::NW][S::PPL];
#define CER_REQUEST(ix, b)                                                                       \
    {                                                                                            \
        const uint4* p_ = reinterpret_cast<const uint4*>(colI + (b)) + lane;                     \
        _Pragma("unroll") for (int W = 0; W < S::NW; ++W)                                        \
            ix[W] = p_[((b) + (uint32_t)W * S::WIN < te ? W : 0) * kWave];                        \
    }
#define CER_BATCH(ix, b)                                                                         \
    bitmap_build<S>(ends, (uint32_t)count + 1u, first, b, bmp, wpre, lane);                      \
    _Pragma("unroll") for (int W = 0; W < S::NW; ++W)                                            \
        if (W == 0 || (b) + (uint32_t)W * S::WIN < te) window_weights<S>(W, bmp, wpre, wts, lane, wl[W]); \
    gemv_batch<S, IdxT, true>(ix, xs, 0u, b, te, wl, acc0, acc1);
            CER_REQUEST(ixa, b0)
            for (;;) {
                const uint32_t b1 = b0 + S::BATCH;
                CER_REQUEST(ixb, b1 < te ? b1 : b0)
                CER_BATCH(ixa, b0)
                if (b1 >= te) break;
                const uint32_t b2 = b1 + S::BATCH;
                CER_REQUEST(ixa, b2 < te ? b2 : b1)
                CER_BATCH(ixb, b1)
                if (b2 >= te) break;
                b0 = b2;
            }
#undef CER_BATCH
#undef CER_REQUEST
        }
        wave_lds_sync();  // the list is rebuilt by the next row
        const float y = wave_sum(acc0 + acc1);
        if (kOneRow && parts > 1u) { y_share = y; break; }
        if (lane == 0) Y[r] = y + t_off;
        if (kOneRow) break;
        first_row = false;
    }
    if (kOneRow && parts > 1u) {  // uniform over the workgroup
        if (lane == 0) s_share[wave] = y_share;
        __syncthreads();
        if (part == 0u && r < row_end && lane == 0) {
            float y = s_share[wave];
            for (uint32_t q = 1; q < parts; ++q) y += s_share[wave + q];
            Y[r] = y + t_off;
        }
    }
}

// Builds the rank table of a handle whose codebook has 2 .. 256 values from its format arrays: one wave per row.
__global__ __launch_bounds__(256) void rank_table_kernel(KView v, uint32_t* __restrict__ tab, uint32_t tab_shift) {
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t r = blockIdx.x * (blockDim.x >> 6) + uniform(threadIdx.x >> 6);
    if (r >= v.m) return;
    const uint2 d0 = v.rowInfo[r], d1 = v.rowInfo[r + 1];
    const uint32_t g0 = d0.x, ng = d1.x - g0;  // at most 255 groups
    const uint32_t words = 1u << tab_shift;
    for (uint32_t w0 = 0; w0 < words; w0 += kWave) {
        const uint32_t word = w0 + lane;
        // the number of the row's groups whose rank is at most `word`: CER numbers its groups by rank (padding groups
        // included), CSER names each group's rank in OmegaI (ascending inside a row)
        uint32_t upto = min(word, ng);
        if (v.cser) {
            upto = 0;
            for (uint32_t j0 = 0; j0 < ng; j0 += kWave) {  // wave-uniform bounds
                const uint32_t mine = j0 + lane < ng ? load_rank(v.omegaI, v.omegaI_bits, g0 + j0 + lane) : kNoEnd;
                const uint32_t nj = min((uint32_t)kWave, ng - j0);
                for (uint32_t j = 0; j < nj; ++j) upto += (uint32_t)__shfl((int)mine, (int)j, kWave) <= word ? 1u : 0u;
            }
        }
        if (word < words) tab[((size_t)r << tab_shift) + word] = v.omegaPtr[g0 + upto];
    }
}

// ------------------------------------------------------------------------------------------------
// batch = 1, values expanded per position (on request)
// ------------------------------------------------------------------------------------------------
//
// The group structure is expanded as in the default batched kernel: per chunk of kGemvExpChunk colI positions the
// value of every position goes to an array in LDS (long groups written by the whole wave, short ones by one lane
// each) and the stream is acc += X[colI[p]] . val[p], lane = position, X staged in LDS.  One wave per row; the index
// loads of a chunk are issued before its expansion starts and run into the next row or the padding behind colI.
// The expansion costs a pass over the groups per chunk and one 2-byte index load per position and lane; the stream
// kernel's bitmap needs neither, which is why this kernel is no longer chosen by the library.

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
// Launch logic
// ------------------------------------------------------------------------------------------------

// LDS the batch-1 kernels may claim dynamically: the device's limit less its few static words.
size_t gemv_lds_budget(const DeviceView& d) { return d.lds_per_block - 256; }

// Whether the stream kernel stages X in LDS for this matrix: whenever it fits beside Omega and the group lists of
// 4 waves (with at least 64 entries each).
bool gemv_stages_x(const DeviceView& d, const MatmulOptions& o) {
    const size_t x_bytes = (((size_t)d.n + 3) & ~(size_t)3) * sizeof(float);
    const size_t om_bytes = d.K <= 4096 ? (((size_t)d.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    const uint32_t gcap = std::max<uint32_t>(1u, (uint32_t)std::min<int64_t>(d.max_row_groups, 1022));
    return (o.flags & kOptXFromGlobal) == 0 &&
           x_bytes + om_bytes + (size_t)4 * ((std::min<uint32_t>(gcap, 64u) + 3) * 8 + 64 * 8) <= gemv_lds_budget(d);
}

template <typename IdxT>
hipError_t launch_gemv(const DeviceView& d, const KView& k, const float* X, float* Y, const float* T, hipStream_t stream,
                       const MatmulOptions& o) {
    const size_t budget = gemv_lds_budget(d);
    const size_t x_bytes = (((size_t)k.n + 3) & ~(size_t)3) * sizeof(float);
    const bool x_in_lds = gemv_stages_x(d, o);
    // codebooks of at most 64 values with X in LDS: the kernel over the rank table (lists of 68 entries, Omega read
    // once per lane from global memory)
    // (its lists have a fixed length: X and the lists of four waves must fit)
    const size_t tab_list_bytes = ((size_t)std::max<uint32_t>(64u, 1u << d.rank_tab_shift) + 4) * 8 + GemvShape<IdxT>::NWORDS * 8;
    const bool use_tab = x_in_lds && d.rank_tab != nullptr && (o.flags & kOptNoRankTable) == 0 && k.m > 0 && k.K >= 2 &&
                         x_bytes + 4 * tab_list_bytes + 256 <= budget;
    const bool omega_in_lds = !use_tab && k.K <= 4096;
    const size_t om_bytes = omega_in_lds ? (((size_t)k.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    // per-wave list of non-empty groups: as long as the longest row needs, at most 1022 entries
    uint32_t gcap = use_tab ? std::max<uint32_t>(64u, 1u << d.rank_tab_shift) + 1u  // lists of max(64, words per record) + 4
                            : std::max<uint32_t>(1u, (uint32_t)std::min<int64_t>(d.max_row_groups, 1022));
    // per wave: the list (a pseudo group, the groups, two sentinels), the batch's bitmap and its word prefix
    auto list_bytes = [&](int waves) {
        return (size_t)waves * ((gcap + 3) * 8 + GemvShape<IdxT>::NWORDS * 8) + (use_tab ? 256u : 0u);  // + counter and sums
    };
    const size_t fixed = (x_in_lds ? x_bytes : 0) + om_bytes;
    // Staging X is what a launch costs a compute unit (about 26 clocks of its vector-memory pipeline per kilobyte), so
    // X should be staged once per compute unit: as many waves per workgroup as the rows spread over all compute units
    // need, at most 16 (a power of two); matrices of few rows get small workgroups on every compute unit.
    // An X of a few kilobytes costs little to stage: workgroups of 4 waves, several per compute unit (measured equal or
    // faster on 2048 x 2048 and 512 x 4608 matrices).
    int waves = 4;
    if (x_in_lds && x_bytes > 24 * 1024) {
        const uint32_t per_unit = (k.m + (uint32_t)d.cus - 1) / (uint32_t)d.cus;
        waves = (int)std::min<uint32_t>(16u, pow2_ceil(std::max<uint32_t>(per_unit, 4u)));
        // long rows (eight windows or more on average) and an X of at most 48 KB: two workgroups of 8 waves per
        // compute unit instead of one of 16 -- X is staged twice, but a wave waits for 7 others instead of 15 before
        // its first gather (the 7-bit layer of 7000 indices per row: 14.3 -> 14.1 us, alternating runs; rows of 1400: no change)
        if (x_bytes <= 48 * 1024 && (uint64_t)d.nnz >= 8ull * GemvShape<IdxT>::WIN * (uint64_t)k.m) waves = std::min(waves, 8);
    }
    // Few rows (at most 2 per compute unit) of at least 3 windows each: a row is shared by 4 or 8 waves, and a
    // workgroup holds as many rows as spread the matrix over all compute units.  Measured against whole rows: 512 x
    // 4608 with 1840 indices per row 4.84 against 5.29 us, 256 x 25088 (1250) 5.2 against 6.8 us, 64 x 4096 (2050)
    // 4.85 against 5.25 us; with 4 or 8 rows per compute unit (1024 x 9216, 2048 x 9216) or rows of 2 windows (512 x
    // 2048) sharing lost 0.2 - 0.6 us (every wave builds the row's group list; 16 waves per compute unit contend).
    uint32_t part_shift = 0, rows_shared = 0;
    if (x_in_lds && (o.flags & kOptRowsWhole) == 0 && k.m > 0 && (uint64_t)k.m <= 2ull * (uint64_t)d.cus &&
        (uint32_t)d.max_row_groups <= gcap) {
        const uint32_t per_unit = pow2_ceil((k.m + (uint32_t)d.cus - 1) / (uint32_t)d.cus);  // 1 or 2
        const uint64_t windows = ((uint64_t)d.nnz / k.m + GemvShape<IdxT>::WIN - 1) / GemvShape<IdxT>::WIN;  // average row
        uint32_t p = windows >= 3 ? std::min<uint32_t>(8u / per_unit, pow2_ceil((uint32_t)std::min<uint64_t>(windows, 8))) : 1u;
        while (p > 1 && fixed + list_bytes((int)(per_unit * p)) > budget) p >>= 1;
        if (p > 1) {
            rows_shared = per_unit;
            while ((1u << part_shift) < p) ++part_shift;
            // idle waves beyond the rows' help to stage a large X (8 KB per wave)
            waves = (int)std::max<uint32_t>(per_unit * p, std::min<uint32_t>(16u, pow2_ceil((uint32_t)(x_bytes / 8192))));
            while (waves > (int)(per_unit * p) && fixed + list_bytes(waves) > budget) waves >>= 1;
        }
    }
    // eight 16-byte loads per thread should cover X (what is left is copied by a plain loop)
    if (x_in_lds) waves = std::max(waves, (int)std::min<uint32_t>(16u, pow2_ceil((uint32_t)((x_bytes / 16 + 511) / 512))));
    while (fixed + list_bytes(waves) > budget && waves > 4) waves >>= 1;
    while (!use_tab && fixed + list_bytes(waves) > budget && gcap > 64) gcap = std::max<uint32_t>(64u, gcap / 2);
    const size_t lds = fixed + list_bytes(waves);
    if (lds > budget) return hipErrorInvalidValue;
    // resident workgroups per CU, limited by LDS and by 32 waves per CU
    size_t per_cu = std::min<size_t>(d.lds_per_block / (lds + 256), (size_t)(32 / waves));
    per_cu = std::max<size_t>(1, std::min<size_t>(per_cu, 8));
    const uint64_t slots = (uint64_t)d.cus * per_cu;
    const uint32_t iters = std::max<uint32_t>((uint32_t)((k.m + slots * waves - 1) / (slots * waves)), 1u);
    // one round of workgroups: no more rows per workgroup than spread the matrix over all compute units (waves
    // without a row only help to stage X)
    uint32_t rows_per_block = rows_shared ? rows_shared : iters * waves;
    if (!rows_shared && iters == 1)
        rows_per_block = std::min<uint32_t>((uint32_t)waves, std::max<uint32_t>(1u, (k.m + (uint32_t)d.cus - 1) / (uint32_t)d.cus));
    const uint32_t blocks = (k.m + rows_per_block - 1) / rows_per_block;
    if (rows_per_block >= (1u << 28)) return hipErrorInvalidValue;
    const bool vec4 = (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && k.n >= 4;
    const bool one = rows_shared != 0 || rows_per_block <= (uint32_t)waves;  // a wave has at most one row
    if (use_tab) {
        using TabKern = void (*)(const uint32_t*, const float*, const float*, const void*, float*, uint32_t, uint32_t, uint32_t,
                                 uint32_t);
        const bool bigx = vec4 && 6ull * (uint64_t)waves * kWave <= (uint64_t)(k.n >> 2);
        // 16-bit indices, rows of more than three windows on average: batches of two windows
        const bool shortb = sizeof(IdxT) == 2 && vec4 && (uint64_t)d.nnz > 3ull * GemvShape<IdxT>::WIN * (uint64_t)k.m;
        TabKern tk = bigx ? (one ? cer_gemv_tab_kernel<IdxT, true, true, true> : cer_gemv_tab_kernel<IdxT, true, false, true>)
                     : vec4 ? (one ? cer_gemv_tab_kernel<IdxT, true, true, false> : cer_gemv_tab_kernel<IdxT, true, false, false>)
                            : (one ? cer_gemv_tab_kernel<IdxT, false, true, false> : cer_gemv_tab_kernel<IdxT, false, false, false>);
        if (shortb)
            tk = bigx ? (one ? cer_gemv_tab_kernel<IdxT, true, true, true, true> : cer_gemv_tab_kernel<IdxT, true, false, true, true>)
                      : (one ? cer_gemv_tab_kernel<IdxT, true, true, false, true> : cer_gemv_tab_kernel<IdxT, true, false, false, true>);
        if (lds > 48 * 1024) {
            static LdsGrant<36> grant;
            const int wslot = sizeof(IdxT) == 1 ? 0 : (sizeof(IdxT) == 2 ? 1 : 2);
            const hipError_t e = grant.ensure(wslot * 12 + (shortb ? 6 : 0) + (bigx ? 4 : (vec4 ? 2 : 0)) + (one ? 1 : 0),
                                              reinterpret_cast<const void*>(tk), budget);
            if (e != hipSuccess) return e;
        }
        {   // the kernel takes LDS address 0 for X: it must not have static LDS in front of the dynamic array
            static std::atomic<int> checked[3][12] = {};
            const int wslot = sizeof(IdxT) == 1 ? 0 : (sizeof(IdxT) == 2 ? 1 : 2);
            std::atomic<int>& c = checked[wslot][(shortb ? 6 : 0) + (bigx ? 4 : (vec4 ? 2 : 0)) + (one ? 1 : 0)];
            if (c.load(std::memory_order_acquire) == 0) {
                hipFuncAttributes fa;
                const hipError_t e = hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(tk));
                if (e != hipSuccess) return e;
                c.store(fa.sharedSizeBytes == 0 ? 1 : 2, std::memory_order_release);
            }
            if (c.load(std::memory_order_acquire) != 1) return hipErrorInvalidDeviceFunction;
        }
        const uint32_t meta = k.K | ((uint32_t)d.rank_tab_shift << 9) | (part_shift << 13) | ((uint32_t)waves << 16);
        hipLaunchKernelGGL(tk, dim3(blocks), dim3(waves * kWave), lds, stream, d.rank_tab, X, k.omega, k.colI, Y, k.n, k.m,
                           rows_per_block, meta);
        return hipGetLastError();
    }
    using Kern = void (*)(const void*, const uint2*, const float*, float*, const uint32_t*, const float*, uint32_t, uint32_t,
                          uint32_t, uint32_t, uint32_t, float, const void*, const float*, int, int);
    Kern kern;
#define CER_GEMV_PICK(CSER, ONE)                                                                 \
    (x_in_lds ? (vec4 ? cer_gemv_kernel<IdxT, true, true, CSER, ONE>                             \
                      : cer_gemv_kernel<IdxT, true, false, CSER, ONE>)                           \
              : cer_gemv_kernel<IdxT, false, false, CSER, ONE>)
    if (k.cser)
        kern = one ? CER_GEMV_PICK(true, true) : CER_GEMV_PICK(true, false);
    else
        kern = one ? CER_GEMV_PICK(false, true) : CER_GEMV_PICK(false, false);
#undef CER_GEMV_PICK
    if (lds > 48 * 1024) {
        static LdsGrant<3 * 12> grant;  // per index width
        const int kslot = (x_in_lds ? (vec4 ? 2 : 1) : 0) + (k.cser ? 3 : 0) + (one ? 6 : 0);
        const int wslot = sizeof(IdxT) == 1 ? 0 : (sizeof(IdxT) == 2 ? 1 : 2);
        const hipError_t e = grant.ensure(wslot * 12 + kslot, reinterpret_cast<const void*>(kern), budget);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, stream, k.colI, k.rowInfo, X, Y, k.omegaPtr, k.omega, k.n,
                       k.m, k.K, rows_per_block | (part_shift << 28), gcap, k.omega0, k.omegaI, T, k.omegaI_bits, omega_in_lds ? 1 : 0);
    return hipGetLastError();
}

// Launch shape of the expansion kernel; waves == 0: X, Omega and the value arrays of four waves do not fit in LDS.
struct GemvExpandPlan {
    int waves = 0;
    uint32_t chunk = 2048;
    size_t lds = 0;
    bool omega_in_lds = false;
};

GemvExpandPlan plan_gemv_expand(const DeviceView& d) {
    GemvExpandPlan p;
    const size_t budget = gemv_lds_budget(d);
    const size_t x_bytes = (((size_t)d.n + 3) & ~(size_t)3) * sizeof(float);
    p.omega_in_lds = d.K <= 4096;
    const size_t om_bytes = p.omega_in_lds ? (((size_t)d.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    p.chunk = d.nnz <= d.m * 384 ? 512u : 2048u;  // by the average row
    const size_t per_wave = (p.chunk + kWave) * sizeof(float);
    // a workgroup that stages a large X should own many rows; a small X leaves room for more, smaller workgroups
    int waves = x_bytes > 40 * 1024 ? 16 : (d.m >= 8192 ? 16 : (d.m >= 4096 ? 8 : 4));
    while (waves > 4 && x_bytes + om_bytes + waves * per_wave > budget) waves >>= 1;
    if (x_bytes + om_bytes + waves * per_wave > budget) return p;
    p.waves = waves;
    p.lds = x_bytes + om_bytes + waves * per_wave;
    return p;
}

// The expansion kernel's plan for this matrix if the caller prefers that kernel and X fits in LDS (waves == 0
// otherwise).  The library itself always takes the stream kernel: alternating measurements on 2048 x 2048 matrices
// with 4 to 256 values and 50 - 99 % zeros, on matrices of 16384 short rows and on the layer shapes show it equal
// or faster everywhere but on 256-value matrices with 90 % zeros or more (6.5 against 6.1 us).
GemvExpandPlan gemv_expand_choice(const DeviceView& d, const MatmulOptions& o) {
    if (o.path == 4) return plan_gemv_expand(d);
    return GemvExpandPlan{};
}

template <typename IdxT>
hipError_t launch_gemv_expand(const DeviceView& d, const KView& k, const GemvExpandPlan& p, const float* X, float* Y,
                              hipStream_t stream) {
    using Kern = void (*)(KView, const float*, float*, uint32_t, int);
    const bool small = p.chunk == 512;
    Kern kern = k.cser ? (small ? cer_gemv_expand_kernel<IdxT, true, 512> : cer_gemv_expand_kernel<IdxT, true, 2048>)
                       : (small ? cer_gemv_expand_kernel<IdxT, false, 512> : cer_gemv_expand_kernel<IdxT, false, 2048>);
    if (p.lds > 48 * 1024) {
        static LdsGrant<12> grant;
        const int wslot = sizeof(IdxT) == 1 ? 0 : (sizeof(IdxT) == 2 ? 1 : 2);
        const hipError_t e = grant.ensure(wslot * 4 + (k.cser ? 1 : 0) + (small ? 2 : 0), reinterpret_cast<const void*>(kern),
                                          gemv_lds_budget(d));
        if (e != hipSuccess) return e;
    }
    const uint32_t rows_per_block = (uint32_t)p.waves;
    const uint32_t blocks = (k.m + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(p.waves * kWave), p.lds, stream, k, X, Y, rows_per_block,
                       p.omega_in_lds ? 1 : 0);
    return hipGetLastError();
}

}  // namespace

int build_rank_table(const DeviceView& d, void* stream) {
    if (!d.rank_tab || d.m <= 0) return (int)hipSuccess;
    const KView k = make_kview(d);
    hipLaunchKernelGGL(rank_table_kernel, dim3((uint32_t)((d.m + 3) / 4)), dim3(256), 0, static_cast<hipStream_t>(stream), k,
                       const_cast<uint32_t*>(d.rank_tab), (uint32_t)d.rank_tab_shift);
    return (int)hipGetLastError();
}

int gemv_path(const DeviceView& d, const MatmulOptions& o) { return gemv_expand_choice(d, o).waves > 0 ? 4 : 0; }

bool gemv_sums_x(const DeviceView& d, const MatmulOptions& o) {
    return gemv_expand_choice(d, o).waves > 0 || gemv_stages_x(d, o);
}

hipError_t launch_gemv_any(const DeviceView& d, const float* X, float* Y, const float* T, hipStream_t stream,
                           const MatmulOptions& o) {
    const KView k = make_kview(d);
    const GemvExpandPlan gx = gemv_expand_choice(d, o);
    if (gx.waves > 0) {
        switch (d.colI_bits) {
            case 8: return launch_gemv_expand<uint8_t>(d, k, gx, X, Y, stream);
            case 16: return launch_gemv_expand<uint16_t>(d, k, gx, X, Y, stream);
            default: return launch_gemv_expand<uint32_t>(d, k, gx, X, Y, stream);
        }
    }
    switch (d.colI_bits) {
        case 8: return launch_gemv<uint8_t>(d, k, X, Y, T, stream, o);
        case 16: return launch_gemv<uint16_t>(d, k, X, Y, T, stream, o);
        default: return launch_gemv<uint32_t>(d, k, X, Y, T, stream, o);
    }
}

}  // namespace cer
