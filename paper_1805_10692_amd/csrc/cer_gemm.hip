// Batch > 1: Y = W.X with W in CER / CSER form, rows of X gathered from L2 (Appendix A-C, Algorithms 3 and 4).
//
// P lanes x V floats cover a tile of batch columns, 64/P indices are gathered per wave instruction (whole
// 128-byte rows of X for the default 32-column tile), two batches of gathers are kept in flight; the indices come
// from one coalesced load per 64 positions and a cross-lane read, several batches ahead; workgroups are numbered
// so that one XCD's L2 sees as few batch tiles of X as possible.  The default kernel expands the group values
// into a per-position array in LDS and multiplies every gathered row by its position's value (no cursor in the
// stream; a multiply-add costs what an add costs); the cursor variant sums a group before its one multiplication.
#include "cer_device.hpp"

namespace cer {
namespace {

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
    const PtrTile pt0 = load_ptr_tile_first(v, cser, g0, g0, min(tg_end0, g0 + (uint32_t)kWave), lane);
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
// kTab (handles of 2 - 64 values, rows whole and in place): the wave finds its row in the rank table -- one record per
// row at a fixed stride, word 0 = the row's first colI position, word k = the end of its group of rank k -- so its first
// memory request brings the row's extent and every group boundary; row_src_ is then the table (otherwise the row
// descriptors), its log2(words per record) sits in the top four bits of ntiles_.
template <typename IdxT, int V, int P, bool kRagged, int kExpChunk = kExpChunkLong, bool kSplit = false, bool kTab = false>
__global__ __launch_bounds__(256) void cer_gemm_expand_kernel(const void* __restrict__ row_src_, const void* __restrict__ colI_,
                                                              const float* __restrict__ X, float* __restrict__ Y, uint32_t L,
                                                              uint32_t ntiles_, uint32_t rowblocks, uint32_t items_per_xcd,
                                                              uint32_t m_, const float* __restrict__ T, KView v, SplitArgs sp) {
    // The first 13 dwords of arguments (plain pointers and integers) arrive in scalar registers with the wave (the
    // library is built with kernel-argument preloading): the row descriptor and the first indices are requested
    // without waiting for a load of the argument block; what else the kernel needs of the matrix (v) comes behind.
    using G = GemmIdx<P>;
    constexpr int S = G::S, U = G::U, KQ = G::KQ, D = G::D;
    constexpr uint32_t PB = G::PB;
    constexpr uint32_t PAD = D * PB;  // the last loop body of a chunk reads (zero) values this far past its end
    constexpr int TW = V * P;
    static_assert(!(kTab && kSplit), "the rank table serves rows that are whole and in place");
    __shared__ float s_val[4][kExpChunk + PAD];
    const uint32_t ntiles = ntiles_ & 0x0FFFFFFFu, tab_shift = ntiles_ >> 28;
    const uint2* rowInfo_ = static_cast<const uint2*>(row_src_);

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
            if (rank >= m_) return;
            r = uniform(sp.order[rank]);
        } else {
            r = rb * 4u + wave;
            if (r >= m_) return;
        }
    }

    const uint32_t sub = lane / P;
    const uint32_t col0 = tile * TW + (lane % P) * V;
    const bool active = col0 < L;
    static_assert(!kRagged || V == 4, "ragged batches are gathered four columns at a time");
    const uint32_t colx = kRagged ? min(col0, L - 4u) : col0;  // ragged: L >= 4 (the launcher sees to it)
    const float* xgather = X + (active ? colx : 0u);
    const IdxT* colI = static_cast<const IdxT*>(colI_);
    float* val = s_val[wave];

    uint32_t g0 = 0, g1 = 0, rs, re;
    PtrTile tab_tile{0u, 0u, 0u};
    if (kTab) {
        const uint32_t last_word = (1u << tab_shift) - 1u;  // at most 63
        const uint32_t rec = static_cast<const uint32_t*>(row_src_)[((size_t)r << tab_shift) + min(lane, last_word)];
        rs = (uint32_t)__builtin_amdgcn_readlane((int)rec, 0);
        re = (uint32_t)__builtin_amdgcn_readlane((int)rec, (int)last_word);
        // lane l holds the group of rank l + 1, which ends where the next lane's begins
        tab_tile.s = rec;
        tab_tile.e = (uint32_t)__builtin_amdgcn_update_dpp((int)rec, (int)rec, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
        if (lane >= last_word) tab_tile.e = tab_tile.s;
        tab_tile.rank = lane + 1u;
    } else {
        const uint2 d0 = rowInfo_[r], d1 = rowInfo_[r + 1];
        g0 = d0.x;
        g1 = d1.x;
        rs = d0.y;
        re = d1.y;
    }
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
        PtrTile p_first = tab_tile;
        if (!kTab) p_first = load_ptr_tile_first(v, cser, g0, gcur, g1, lane);
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
        auto expand_tile = [&](const PtrTile& p) {
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
        };
        if (kTab) {
            expand_tile(p_first);  // the record holds every group of the row
        } else {
            for (uint32_t gt = gcur; gt < g1; gt += kWave) {
                const PtrTile p = gt == g_first ? p_first : load_ptr_tile(v, cser, g0, gt, g1, lane);
                expand_tile(p);
                // groups of this tile that end inside the chunk are done with
                const uint32_t done = (uint32_t)__popcll(__ballot(gt + lane < g1 && p.e <= c1));
                gcur = gt + done;
                if (done < (uint32_t)kWave) break;  // the next group reaches beyond the chunk (or the row is finished)
            }
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
// Launch logic
// ------------------------------------------------------------------------------------------------

// The kernel that expands the group values per position is the default: measured on MI355X it beats the cursor
// kernel on every workload (1.05 - 1.2 x on the layer shapes, up to 2 x on rows of many short groups); the caller's
// options can ask for the cursor kernel.
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
    hipLaunchKernelGGL(kern, dim3((uint32_t)blocks), dim3(256), 0, stream, k.rowInfo, k.colI, X, Y, L, ntiles, rowblocks, ipx,
                       k.m, T, k, sp);
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
                          const SplitArgs& sp, bool expand, bool short_rows = false, bool no_tab = false) {
    constexpr uint32_t TW = V * P;
    const uint32_t ntiles = (L + TW - 1) / TW;
    const uint32_t rowblocks = (k.m + 3) / 4;
    const uint64_t nitems = (uint64_t)ntiles * rowblocks;
    if (nitems > 0x7FFFFFFFull / 8) return hipErrorInvalidValue;
    const uint32_t ipx = (uint32_t)((nitems + 7) / 8);
    if (expand) {
        if (sp.order) {
            if (TW == 32 && V == 4 && short_rows)
                return launch_expand_split(cer_gemm_expand_kernel<IdxT, 4, 8, false, kExpChunkShort, true>, k, X, Y, T, L,
                                           ntiles, rowblocks, ipx, sp, stream);
            return launch_expand_split(cer_gemm_expand_kernel<IdxT, V, P, false, kExpChunkLong, true>, k, X, Y, T, L, ntiles,
                                       rowblocks, ipx, sp, stream);
        }
        // handles of 2 - 64 values, batches of whole 16-byte pieces: the row's extent and group boundaries from the rank
        // table (records of at most 64 words), one trip to memory instead of two before the expansion can start
        const bool tab = V == 4 && k.rank_tab != nullptr && k.K >= 2 && k.rank_tab_shift >= 1 && k.rank_tab_shift <= 6 &&
                         ntiles < (1u << 28) && !no_tab;
        const uint32_t ntiles_tab = ntiles | ((uint32_t)k.rank_tab_shift << 28);
        if (TW == 32 && V == 4 && short_rows) {
            if (tab)
                hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, 8, false, kExpChunkShort, false, true>), dim3(ipx * 8), dim3(256),
                                   0, stream, k.rank_tab, k.colI, X, Y, L, ntiles_tab, rowblocks, ipx, k.m, T, k, SplitArgs{});
            else
                hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, 8, false, kExpChunkShort>), dim3(ipx * 8), dim3(256), 0, stream,
                                   k.rowInfo, k.colI, X, Y, L, ntiles, rowblocks, ipx, k.m, T, k, SplitArgs{});
        } else if (tab && V == 4) {
            hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, (V == 4 ? P : 8), false, kExpChunkLong, false, true>), dim3(ipx * 8),
                               dim3(256), 0, stream, k.rank_tab, k.colI, X, Y, L, ntiles_tab, rowblocks, ipx, k.m, T, k, SplitArgs{});
        } else {
            hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, V, P, false>), dim3(ipx * 8), dim3(256), 0, stream, k.rowInfo, k.colI,
                               X, Y, L, ntiles, rowblocks, ipx, k.m, T, k, SplitArgs{});
        }
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
        hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, 8, true, kExpChunkShort>), dim3(ipx * 8), dim3(256), 0, stream,
                           k.rowInfo, k.colI, X, Y, L, ntiles, rowblocks, ipx, k.m, T, k, SplitArgs{});
    else
        hipLaunchKernelGGL((cer_gemm_expand_kernel<IdxT, 4, P, true>), dim3(ipx * 8), dim3(256), 0, stream, k.rowInfo, k.colI, X,
                           Y, L, ntiles, rowblocks, ipx, k.m, T, k, SplitArgs{});
    return hipGetLastError();
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
                       const SplitArgs& sp, bool short_rows, const MatmulOptions& o) {
    const bool expand = (o.flags & kOptSumThenMultiply) == 0;
    const bool no_tab = (o.flags & kOptNoRankTable) != 0;
    const bool vec4 = (L % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0) &&
                      ((reinterpret_cast<uintptr_t>(Y) & 15u) == 0) && ((reinterpret_cast<uintptr_t>(T) & 15u) == 0);
    if (vec4) {
        // tile width: all of L up to 32 columns, 32 beyond: one gather = one 128-byte line of an X row, and a
        // wider batch gives more waves (measured on MI355X: 32 beats 16, 64, 128 and 256 at L = 32, 64, 3136)
        uint32_t tw = std::min<uint32_t>(pow2_ceil(L), 32u);
        tw = std::max<uint32_t>(tw, 8u);  // 4-column tiles (64 distinct rows per gather instruction) measured 1.4 - 3 x slower
        if (L > 32) tw = pick_wide_tile(L, k.m, X, 128u);
        if (o.tile_cols > 0) tw = (uint32_t)o.tile_cols;
        switch (tw) {
            case 4: return launch_gemm_vp<IdxT, 4, 1>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            case 8: return launch_gemm_vp<IdxT, 4, 2>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            case 16: return launch_gemm_vp<IdxT, 4, 4>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            case 32: return launch_gemm_vp<IdxT, 4, 8>(k, X, Y, T, L, stream, sp, expand, short_rows, no_tab);
            case 64: return launch_gemm_vp<IdxT, 4, 16>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            case 128: return launch_gemm_vp<IdxT, 4, 32>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            case 256: return launch_gemm_vp<IdxT, 4, 64>(k, X, Y, T, L, stream, sp, expand, false, no_tab);
            default: return hipErrorInvalidValue;
        }
    }
    if (L >= 4 && expand && (o.flags & kOptOneColumnPerLane) == 0) {
        // ragged width or 4-byte aligned buffers: still four columns per lane
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
        case 1: case 2: return launch_gemm_vp<IdxT, 1, 2>(k, X, Y, T, L, stream, sp, expand);
        case 4: return launch_gemm_vp<IdxT, 1, 4>(k, X, Y, T, L, stream, sp, expand);
        case 8: return launch_gemm_vp<IdxT, 1, 8>(k, X, Y, T, L, stream, sp, expand);
        case 16: return launch_gemm_vp<IdxT, 1, 16>(k, X, Y, T, L, stream, sp, expand);
        case 32: return launch_gemm_vp<IdxT, 1, 32>(k, X, Y, T, L, stream, sp, expand);
        default: return launch_gemm_vp<IdxT, 1, 64>(k, X, Y, T, L, stream, sp, expand);
    }
}

}  // namespace

hipError_t launch_gemm_any(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                           const MatmulOptions& o) {
    const KView k = make_kview(d);
    // 512-position value chunks for matrices of short rows (32-column tiles); the options can force either size
    const bool short_rows = (o.flags & kOptShortChunks) != 0 || ((o.flags & kOptLongChunks) == 0 && d.nnz <= d.m * 384);
    SplitArgs sp;  // kOptRowsWhole: rows in their own order, long rows whole
    if (d.row_order && (o.flags & kOptRowsWhole) == 0) {
        sp.order = static_cast<const uint32_t*>(d.row_order);
        sp.parts = static_cast<const uint4*>(d.split_parts);
        sp.rows = static_cast<const uint4*>(d.split_rows);
        sp.nparts = d.n_split_parts;
        sp.nrows = d.n_split_rows;
        sp.len = d.split_len;
        sp.min = d.split_min;
    }
    switch (d.colI_bits) {
        case 8: return launch_gemm<uint8_t>(k, X, Y, T, L, stream, sp, short_rows, o);
        case 16: return launch_gemm<uint16_t>(k, X, Y, T, L, stream, sp, short_rows, o);
        default: return launch_gemm<uint32_t>(k, X, Y, T, L, stream, sp, short_rows, o);
    }
}

}  // namespace cer
