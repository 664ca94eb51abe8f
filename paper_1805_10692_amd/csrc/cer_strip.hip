// Batch > 1 with strips of X resident in LDS: the reuse of input elements that Section V-C of the paper names as the
// missing optimisation, in its column-blocked form.
//
// The kernels that gather rows of X from L2 are bound by the compute unit's vector-memory pipeline (about 26 clocks
// per wave instruction of 1 KB, i.e. 40 bytes per clock); LDS delivers 128 bytes per clock.  Here the input is cut
// into equally long strips of at most 1024 consecutive rows; a workgroup copies one strip of one tile of 32 batch columns into LDS
// (128 KB, rows of 128 bytes) and serves from it every indexed element of its rows of W whose column falls into the
// strip.  The format orders a row's indices by value, then column, so a strip's share of a row is scattered over
// the row's groups: the handle carries a DERIVED strip-major index (built once by cer_prepare_strips from the format
// arrays), whose 16-bit entries hold the rank of the element's value (6 bits: codebooks of at most 64 values) and
// the column inside the strip (10 bits).  The entries of one (strip, row) are padded to a multiple of eight -- a
// chunk of 16 bytes -- with entries of rank 0, whose weight Omega[0] - Omega[0] is zero; the pointers count chunks.
// Every element is multiplied by its own value, so the fragmentation of the groups does not matter.
//
// Lanes: a quad (4 lanes) serves one entry at a time: 32 bytes = 8 batch columns per lane, read with two 16-byte LDS
// reads -- lane j takes the pieces j and j + 4 of the entry's 128-byte row, even quads the lower piece first, odd
// quads the upper one, so that the two quads that share an LDS cycle touch different banks.  All 4 lanes load the same
// chunk, so the entries reach them without a cross-lane operation; the weights of a chunk's eight entries are looked
// up once per chunk (lane j those of entries j and j + 4, from a table in LDS that is addressed by the entry's top
// byte: rank and the two top column bits) and handed to the quad by a DPP broadcast per entry.  Per entry and lane:
// 4 address and broadcast instructions, 2 LDS reads, 8 multiply-adds.
// Work: a workgroup's chunks are dealt to its 256 workers (quads) in equal contiguous ranges, whatever rows they
// belong to; a worker writes the rows that begin and end inside its range itself, keeps back the row it ends but did
// not begin, and leaves what it summed behind its last row end as its tail; after the stream the kept-back rows are
// completed from the tails, in worker order (deterministic).  Three chunks are in flight per worker; the ends of the
// workgroup's rows are staged in LDS.  Each (strip, row) leaves a partial sum; a second kernel adds the strips'
// partial sums in strip order and the constant term of a non-zero most frequent value (Appendix A-A1).
#include "cer_device.hpp"

namespace cer {
namespace {

constexpr uint32_t kStripTile = 32;                               // batch columns per tile: one 128-byte row per entry
constexpr uint32_t kStripBytes = kStripRows * kStripTile * 4u;    // the strip in LDS
constexpr uint32_t kStripWtsBytes = 1024;                         // 256 weights in front of it (LDS address 0)
constexpr double kStripRoundUs = 0.85;                             // one chunk per worker, 16 waves per compute unit
constexpr uint32_t kStripMaxRows = 3072;                          // rows of W per workgroup (their ends sit in LDS)

typedef float F4 __attribute__((ext_vector_type(4)));
typedef const F4 __attribute__((address_space(3))) * LdsF4Ptr;
typedef const float __attribute__((address_space(3))) * LdsF1Ptr;

// The value of lane kLane of the lane's quad.
template <int kLane>
__device__ __forceinline__ float quad_broadcast(float w) {
    // (every lane of a quad is a valid source: with bound_ctrl set the destination needs no previous value)
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(w), kLane * 0x55 /* quad_perm:[k,k,k,k] */, 0xF, 0xF, true));
}

// The weights of the two entries of a chunk that lane j of a quad looks up (entries j and j + 4): the entry's top byte
// x 4 is the LDS address of its weight.  half_shift = 16 (j & 1), upper_pair = j & 2.
__device__ __forceinline__ void chunk_weights(const uint4& q, uint32_t half_shift, bool upper_pair, float& w_lo, float& w_hi) {
    uint32_t two = 2u;
    asm("" : "+v"(two));  // the shift count in a vector register (sub-dword forms take no constants)
    const uint32_t d_lo = (upper_pair ? q.y : q.x) >> half_shift, d_hi = (upper_pair ? q.w : q.z) >> half_shift;
    uint32_t a_lo, a_hi;
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(a_lo) : "v"(two), "v"(d_lo));
    asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(a_hi) : "v"(two), "v"(d_hi));
    w_lo = *reinterpret_cast<LdsF1Ptr>((uintptr_t)a_lo);
    w_hi = *reinterpret_cast<LdsF1Ptr>((uintptr_t)a_hi);
}

// Entry kEntry of a chunk: its 128-byte row of the strip (this lane's two pieces) times its weight.  xbase = the LDS
// address of the lane's first piece inside row 0 of the strip; the second piece is 64 bytes above or below it.
template <int kEntry, bool kHalf>
__device__ __forceinline__ void strip_entry(const uint4& q, uint32_t xbase, float w_lo, float w_hi, F4& acc0, F4& acc1) {
    const uint32_t d = kEntry < 2 ? q.x : (kEntry < 4 ? q.y : (kEntry < 6 ? q.z : q.w));
    uint32_t c, xa;  // written out: one bit-field extract and one shift-add
    if (kEntry & 1) asm("v_bfe_u32 %0, %1, 16, 10" : "=v"(c) : "v"(d));
    else asm("v_bfe_u32 %0, %1, 0, 10" : "=v"(c) : "v"(d));
    asm("v_lshl_add_u32 %0, %1, 7, %2" : "=v"(xa) : "v"(c), "v"(xbase));
    const F4 x0 = *reinterpret_cast<LdsF4Ptr>((uintptr_t)xa);
    const float w = quad_broadcast<kEntry & 3>(kEntry < 4 ? w_lo : w_hi);
    acc0.x = fmaf(w, x0.x, acc0.x); acc0.y = fmaf(w, x0.y, acc0.y);
    acc0.z = fmaf(w, x0.z, acc0.z); acc0.w = fmaf(w, x0.w, acc0.w);
    if (!kHalf) {
        const F4 x1 = *reinterpret_cast<LdsF4Ptr>((uintptr_t)(xa ^ 64u));
        acc1.x = fmaf(w, x1.x, acc1.x); acc1.y = fmaf(w, x1.y, acc1.y);
        acc1.z = fmaf(w, x1.z, acc1.z); acc1.w = fmaf(w, x1.w, acc1.w);
    }
}

// One chunk: eight entries.  kHalf: a batch of at most 16 columns -- one piece per lane (the 64 bytes of a row are
// stored twice in its 128 bytes of LDS, even quads read the lower copy, odd quads the upper one).
template <bool kHalf>
__device__ __forceinline__ void strip_chunk(const uint4& q, uint32_t xbase, uint32_t half_shift, bool upper_pair, F4& acc0,
                                            F4& acc1) {
    float w_lo, w_hi;
    chunk_weights(q, half_shift, upper_pair, w_lo, w_hi);
    strip_entry<0, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1); strip_entry<1, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1);
    strip_entry<2, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1); strip_entry<3, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1);
    strip_entry<4, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1); strip_entry<5, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1);
    strip_entry<6, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1); strip_entry<7, kHalf>(q, xbase, w_lo, w_hi, acc0, acc1);
}

// chunks: the strip-major index, 16 bytes per chunk, closed by one chunk of zeros (index zero_chunk);
// sptr[s (m + 1) + r] = first chunk of (strip s, row r).
// part: [strip][m][L rounded up to 4] partial sums.  kHalf: L <= 16 (one tile of at most four 16-byte pieces per row).
// kAlignedX: L is a multiple of 4 and X is 16-byte aligned (otherwise the pieces of X are read from 4-byte aligned
// addresses, the last piece of a row element by element).
template <bool kHalf, bool kAlignedX>
__global__ __launch_bounds__(1024) void cer_strip_kernel(const uint4* __restrict__ chunks, const uint32_t* __restrict__ sptr,
                                                         const float* __restrict__ X, float* __restrict__ part,
                                                         const float* __restrict__ omega, uint32_t m, uint32_t n, uint32_t L,
                                                         uint32_t K, uint32_t ntiles, uint32_t nsplit,
                                                         uint32_t rows_per_split, uint32_t zero_chunk, uint32_t strip_rows) {
    // LDS: [256 weights][strip: rows of 8 x 16 bytes; after the stream: one partial row sum per worker][ends of the
    // workgroup's rows, in chunks]; no static LDS, so the weight of an entry sits at LDS address 4 x (its top byte).
    extern __shared__ __align__(16) unsigned char strip_smem[];
    float* s_w = reinterpret_cast<float*>(strip_smem);
    F4* xs4 = reinterpret_cast<F4*>(strip_smem + kStripWtsBytes);
    F4* s_tail = xs4;
    uint32_t* s_end = reinterpret_cast<uint32_t*>(strip_smem + kStripWtsBytes + kStripBytes);
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t split = blockIdx.x % nsplit, tile = (blockIdx.x / nsplit) % ntiles, s = blockIdx.x / (nsplit * ntiles);
    const uint32_t c0 = s * strip_rows, rows_here = min(strip_rows, n - c0);
    const uint32_t r_begin = min(m, split * rows_per_split), rows = min(m, r_begin + rows_per_split) - r_begin;
    const uint32_t* sp = sptr + (size_t)s * (m + 1) + r_begin;
    const F4* X4 = reinterpret_cast<const F4*>(X);
    const uint32_t row_f4 = (L + 3u) >> 2;  // 16-byte pieces per row of X and of the partial sums (the last one may be partial)
    const uint32_t tile_f4 = min(8u, row_f4 - tile * 8u);  // ... of this tile: fewer than 8 in a ragged last tile
    const uint32_t pieces = rows_here * 8u;

    // (1) Everything is requested at once, all loads unconditional: the ends of the workgroup's rows and Omega first,
    //     then the strip of this tile of batch columns (8 threads copy one 128-byte row, eight loads per thread).
    static_assert(kStripMaxRows + 1 <= 4 * 1024, "four row ends per thread");
    uint32_t er[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) er[k] = sp[min((uint32_t)k * 1024u + threadIdx.x, rows)];
    const float om_r = omega[min(threadIdx.x >> 2, K - 1u)], om_0 = omega[0];
    __builtin_amdgcn_sched_barrier(0);
    F4 xr[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t i = min((uint32_t)k * 1024u + threadIdx.x, pieces - 1u);
        // the pieces of the last tile that lie behind the batch's last column re-read the tile's first piece; a row of
        // at most four pieces is stored twice
        const uint32_t piece = kHalf ? (i & 3u) : (i & 7u);
        const uint32_t col = (tile * 8u + (piece < tile_f4 ? piece : 0u)) * 4u;  // the piece's first batch column
        if (kAlignedX) {
            xr[k] = X4[((size_t)(c0 + (i >> 3)) * L + col) >> 2];
        } else {
            const float* px = X + (size_t)(c0 + (i >> 3)) * L + col;
            if (col + 4u <= L) {
                typedef float F4u __attribute__((ext_vector_type(4), aligned(4)));
                const F4u t = *reinterpret_cast<const F4u*>(px);
                xr[k] = F4{t.x, t.y, t.z, t.w};
            } else {  // the row's last, partial piece
                xr[k] = F4{px[0], col + 1u < L ? px[1] : 0.f, col + 2u < L ? px[2] : 0.f, 0.f};
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t i = (uint32_t)k * 1024u + threadIdx.x;
        if (i <= rows) s_end[i] = er[k];
    }
    if (threadIdx.x < 256u) s_w[threadIdx.x] = (threadIdx.x >> 2) < K ? om_r - om_0 : 0.f;
    __syncthreads();

    // (2) While the strip is on its way: the workgroup's chunks [C0, C1) are dealt to its 256 workers (quads) in equal
    //     contiguous ranges [ca, cb), whatever rows they belong to.  A worker owns the rows that END inside (ca, cb]
    //     (worker 0 also those that end at C0: empty rows in front); its first row is found by a binary search over
    //     the row ends.
    const uint32_t j = lane & 3u, odd = (lane >> 2) & 1u, w = wave * 16u + (lane >> 2);
    // the lane's pieces of a row (first and second read), and where its first read finds them in the row's 128 bytes
    const uint32_t p0 = kHalf ? j : j + 4u * odd, p1 = kHalf ? 8u : j + 4u * (1u - odd);
    const uint32_t xbase = kStripWtsBytes + (j + 4u * odd) * 16u;
    const uint32_t half_shift = 16u * (j & 1u);
    const bool upper_pair = (j & 2u) != 0u;
    const uint32_t C0 = s_end[0], C1 = s_end[rows];
    F4* out0 = reinterpret_cast<F4*>(part) + ((size_t)s * m + r_begin) * row_f4 + tile * 8u;
    if (C1 == C0) {  // uniform over the workgroup: no row has an element in this strip
        for (uint32_t i = threadIdx.x; i < rows * 8u; i += 1024u)
            if ((i & 7u) < tile_f4) out0[(size_t)(i >> 3) * row_f4 + (i & 7u)] = F4{0.f, 0.f, 0.f, 0.f};
        return;
    }
    const uint32_t per = (C1 - C0 + 255u) >> 8;
    const uint32_t ca = min(C1, C0 + w * per), cb = min(C1, ca + per);
    uint32_t r0 = 0;
    {
        uint32_t hi = w == 0u ? 0u : rows;
#pragma unroll 1
        while (__ballot(r0 < hi) != 0ull) {
            const uint32_t mid = (r0 + hi) >> 1;
            const bool later = s_end[min(mid + 1u, rows)] > ca;
            if (r0 < hi) {
                if (later) hi = mid; else r0 = mid + 1u;
            }
        }
    }
    // generator: the worker's next iterations -- a chunk (flag bit 0: the worker is still at work), the end of one
    // row (bit 1), or both.  Free of branches, and every load is issued unconditionally (an iteration without a chunk
    // reads the chunk of zeros behind the index: entries of rank 0, weight zero), so that the waits for the three
    // chunks in flight stay exact.  gnext = end of the row behind the current one, read from LDS an iteration early.
    uint32_t gcr = r0, gbase = ca, gce = s_end[min(r0 + 1u, rows)], gnext = s_end[min(r0 + 2u, rows)];
    auto gen = [&](uint4& q, uint32_t& f) {
        const bool has = gbase < min(gce, cb);
        q = chunks[has ? gbase : zero_chunk];
        gbase += has ? 1u : 0u;
        const bool ends = gbase == gce && gcr < rows && gce <= cb;
        f = ((has || ends) ? 1u : 0u) | (ends ? 2u : 0u);
        gce = ends ? gnext : gce;
        gcr += ends ? 1u : 0u;
        gnext = s_end[min(gcr + 2u, rows)];
    };
    uint4 qa, qb, qc;
    uint32_t fa, fb, fc;
    gen(qa, fa);
    gen(qb, fb);
    __builtin_amdgcn_sched_barrier(0);

    // (3) the strip goes to LDS
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t i = (uint32_t)k * 1024u + threadIdx.x;
        if (i < pieces) xs4[i] = xr[k];
    }
    __syncthreads();

    // (4) the stream.  A row that began in an earlier worker's range is kept back (at most one per worker: the first
    //     it ends); what a worker has summed behind its last row end is its tail.
    const F4 zero4 = F4{0.f, 0.f, 0.f, 0.f};
    F4 acc0 = zero4, acc1 = zero4, head0 = zero4, head1 = zero4;
    uint32_t cr = r0, cs = s_end[min(r0, rows)];  // the consumer's row and where it starts
    uint32_t head_row = 0xFFFFFFFFu, head_start = 0u;
    F4* orow = out0 + (size_t)cr * row_f4;  // where the consumer's row goes
    auto consume = [&](const uint4& q, uint32_t f) {
        strip_chunk<kHalf>(q, xbase, half_shift, upper_pair, acc0, acc1);
        if (f & 2u) {
            // the row a worker ends but did not begin (once per worker at most) is kept back: a branch the wave skips
            const bool kept = cs < ca;
            if (__ballot(kept) != 0ull) {
                if (kept) {
                    head0 = acc0;
                    head1 = acc1;
                    head_row = cr;
                    head_start = cs;
                }
            }
            if (!kept) {
                if (p0 < tile_f4) orow[p0] = acc0;
                if (p1 < tile_f4) orow[p1] = acc1;
            }
            acc0 = zero4;
            acc1 = zero4;
            ++cr;
            orow += row_f4;
            cs = s_end[min(cr, rows)];
        }
    };
    for (;;) {
        gen(qc, fc);
        if (__ballot(fa != 0u) == 0ull) break;
        consume(qa, fa);
        gen(qa, fa);
        if (__ballot(fb != 0u) == 0ull) break;
        consume(qb, fb);
        gen(qb, fb);
        if (__ballot(fc != 0u) == 0ull) break;
        consume(qc, fc);
    }

    // (5) rows shared by several workers: the worker that ends the row adds, in worker order, the tails of the worker
    //     the row began in and of those it runs through (they end no row: their tail is all they summed) to its own
    //     sum.  The tails take the place of the strip, which no worker reads any more.
    __syncthreads();
    s_tail[w * 8u + p0] = acc0;
    if (!kHalf) s_tail[w * 8u + p1] = acc1;
    __syncthreads();
    if (head_row != 0xFFFFFFFFu) {
        uint32_t v = (head_start - C0) / per;  // the worker whose range holds the row's first chunk
        const uint32_t p1r = kHalf ? p0 : p1;  // (one piece per lane: the second sum stays unused)
        F4 sum0 = s_tail[v * 8u + p0], sum1 = s_tail[v * 8u + p1r];
        for (++v; v < w; ++v) {
            const F4 t0 = s_tail[v * 8u + p0], t1 = s_tail[v * 8u + p1r];
            sum0.x += t0.x; sum0.y += t0.y; sum0.z += t0.z; sum0.w += t0.w;
            sum1.x += t1.x; sum1.y += t1.y; sum1.z += t1.z; sum1.w += t1.w;
        }
        sum0.x += head0.x; sum0.y += head0.y; sum0.z += head0.z; sum0.w += head0.w;
        sum1.x += head1.x; sum1.y += head1.y; sum1.z += head1.z; sum1.w += head1.w;
        if (p0 < tile_f4) out0[(size_t)head_row * row_f4 + p0] = sum0;
        if (p1 < tile_f4) out0[(size_t)head_row * row_f4 + p1] = sum1;
    }
}

// Y[r][:] = sum over strips of part[s][r][:]  (+ Omega[0] . T[:]), in strip order.  One thread per 16-byte piece of a row
// of the partial sums; kAlignedY: L is a multiple of 4 and Y is 16-byte aligned (otherwise Y and T are accessed element
// by element).
template <bool kAlignedY>
__global__ __launch_bounds__(256) void cer_strip_sum_kernel(const float* __restrict__ part, float* __restrict__ Y,
                                                            const float* __restrict__ T, float omega0, uint32_t nstrips,
                                                            uint64_t plane_f4, uint32_t row_f4, uint32_t L) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= plane_f4) return;
    const F4* p = reinterpret_cast<const F4*>(part) + i;
    F4 a = F4{0.f, 0.f, 0.f, 0.f};
    // eight planes requested at a time, added in strip order
    uint32_t s = 0;
    for (; s + 8 <= nstrips; s += 8) {
        F4 b[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) b[k] = p[(uint64_t)(s + k) * plane_f4];
#pragma unroll
        for (int k = 0; k < 8; ++k) { a.x += b[k].x; a.y += b[k].y; a.z += b[k].z; a.w += b[k].w; }
    }
    for (; s < nstrips; ++s) {
        const F4 b = p[(uint64_t)s * plane_f4];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    if (kAlignedY) {
        if (omega0 != 0.f) {
            const F4 t = reinterpret_cast<const F4*>(T)[i % row_f4];
            a.x = fmaf(omega0, t.x, a.x); a.y = fmaf(omega0, t.y, a.y);
            a.z = fmaf(omega0, t.z, a.z); a.w = fmaf(omega0, t.w, a.w);
        }
        reinterpret_cast<F4*>(Y)[i] = a;
    } else {
        const uint64_t row = i / row_f4;
        const uint32_t col = (uint32_t)(i - row * row_f4) * 4u;
        const float o[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (uint32_t e = 0; e < 4; ++e)
            if (col + e < L) Y[row * L + col + e] = omega0 != 0.f ? fmaf(omega0, T[col + e], o[e]) : o[e];
    }
}

constexpr size_t strip_lds_bytes(uint32_t rows) {
    return (size_t)kStripWtsBytes + kStripBytes + 4u * ((size_t)rows + 1u);
}

}  // namespace

bool strip_applicable(const DeviceView& d, const float*, const float*, uint32_t L) {
    return d.strip_idx != nullptr && d.n_strips > 0 && L >= 2u && d.m > 0 &&
           d.lds_per_block >= strip_lds_bytes(kStripMaxRows) + 512;
}

// Launch shape of the strip kernel for a batch of L columns, and a rough duration.
//   * One workgroup per compute unit holds 128 KB of LDS, so the (strip, tile) pairs are split over the rows into
//     about as many workgroups as there are compute units (never more than kStripMaxRows rows each).
//   * Duration: a worker's chunks (the workgroup's chunks / 256) x 0.85 us (one chunk per worker with 16 waves on a
//     compute unit) + 7 us for the staging of the strip, the search and the shared rows, per round of workgroups;
//     the launches; the second kernel reads strips x m x L partial sums.  Measured on MI355X / this estimate:
//     AlexNet-fc6 shape batch 32 / 128: 25.3 / 61.4 us (25.9 / 62.6), VGG-fc6 shape batch 32 / 64 / 128: 33.1 / 44.8 /
//     78.0 us (30.7 / 47.3 / 92), 3x3 convolution shape batch 3136: 209 us (215).
StripPlan plan_strip(const DeviceView& d, uint32_t L) {
    StripPlan p;
    const uint32_t m = (uint32_t)d.m;
    p.ntiles = (L + kStripTile - 1) / kStripTile;
    const uint64_t base = (uint64_t)d.n_strips * p.ntiles;
    uint32_t nsplit = (uint32_t)std::max<uint64_t>(1, (uint64_t)d.cus / std::max<uint64_t>(base, 1));
    nsplit = std::max(nsplit, (m + kStripMaxRows - 1) / kStripMaxRows);
    nsplit = std::min(nsplit, std::max(m, 1u));
    p.rows_per_split = (m + nsplit - 1) / nsplit;
    p.nsplit = (m + p.rows_per_split - 1) / std::max(p.rows_per_split, 1u);
    p.blocks = base * p.nsplit;
    const double chunks_per_row = (double)d.strip_chunks / std::max(1.0, (double)d.n_strips * (double)m);
    const double rounds = std::ceil((double)p.rows_per_split * chunks_per_row / 256.0);
    const double wg_rounds = std::ceil((double)p.blocks / std::max(d.cus, 1));
    const double partial_bytes = (double)d.n_strips * m * ((L + 3u) & ~3u) * 4.0;
    // short rows: some quad of a wave ends a row in nearly every iteration, and the whole wave walks through that branch
    const double per_round = (L <= 16u ? 0.6 : 1.0) * kStripRoundUs * (1.0 + 1.5 / std::max(chunks_per_row, 1.0));
    p.est_us = wg_rounds * (rounds * per_round + 7.0) + 3.0 + (3.0 + 2.0 * partial_bytes / 5e6);
    // workgroups with next to nothing to stream (2048 x 2048 cells: 16 rows each) measure 17 - 21 us whatever they hold
    if (rounds < 8.0) p.est_us += 6.0;
    // the library itself never asks for more than 1 GiB of partial sums (as for the decoded matrix of the dense route)
    if (partial_bytes > (double)(1ull << 30)) p.est_us = 1e12;
    return p;
}

hipError_t launch_strip(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream) {
    const uint32_t m = (uint32_t)d.m, n = (uint32_t)d.n;
    const StripPlan sp = plan_strip(d, L);
    if (sp.blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    float* part = nullptr;
    const uint32_t row_f4 = (L + 3u) / 4u;
    const size_t part_bytes = (size_t)d.n_strips * m * row_f4 * 16u;
    hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&part), part_bytes, stream);
    if (e != hipSuccess) return e;
    static LdsGrant<4> grant;
    const bool half = L <= 16u;
    const bool aligned_x = L % 4u == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0;
    const bool aligned_y = L % 4u == 0 && (reinterpret_cast<uintptr_t>(Y) & 15u) == 0 &&
                           (T == nullptr || (reinterpret_cast<uintptr_t>(T) & 15u) == 0);
    auto kern = half ? (aligned_x ? cer_strip_kernel<true, true> : cer_strip_kernel<true, false>)
                     : (aligned_x ? cer_strip_kernel<false, true> : cer_strip_kernel<false, false>);
    e = grant.ensure((half ? 2 : 0) + (aligned_x ? 1 : 0), reinterpret_cast<const void*>(kern), strip_lds_bytes(kStripMaxRows));
    if (e == hipSuccess) {
        hipLaunchKernelGGL(kern, dim3((uint32_t)sp.blocks), dim3(1024), strip_lds_bytes(sp.rows_per_split), stream,
                           static_cast<const uint4*>(d.strip_idx), d.strip_ptr, X, part, d.omega, m, n, L, (uint32_t)d.K,
                           sp.ntiles, sp.nsplit, sp.rows_per_split, (uint32_t)d.strip_chunks, d.strip_rows);
        e = hipGetLastError();
    }
    if (e == hipSuccess) {
        const uint64_t plane_f4 = (uint64_t)m * row_f4;
        const dim3 grid((uint32_t)((plane_f4 + 255) / 256));
        if (aligned_y)
            hipLaunchKernelGGL(cer_strip_sum_kernel<true>, grid, dim3(256), 0, stream, part, Y, T, d.omega0, d.n_strips, plane_f4,
                               row_f4, L);
        else
            hipLaunchKernelGGL(cer_strip_sum_kernel<false>, grid, dim3(256), 0, stream, part, Y, T, d.omega0, d.n_strips, plane_f4,
                               row_f4, L);
        e = hipGetLastError();
    }
    const hipError_t f = (hipError_t)temp_free(part, stream);
    return e == hipSuccess ? f : e;
}

}  // namespace cer
