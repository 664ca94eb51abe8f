// Batch > 1 with strips of X resident in LDS: the reuse of input elements that Section V-C of the paper names as the
// missing optimisation, in its column-blocked form.
//
// The kernels that gather rows of X from L2 are bound by the compute unit's vector-memory pipeline (about 26 clocks
// per wave instruction of 1 KB, i.e. 40 bytes per clock); LDS delivers 128 bytes per clock.  Here the input is cut
// into strips of 1024 consecutive rows; a workgroup copies one strip of one tile of 32 batch columns into LDS
// (128 KB, rows of 128 bytes) and serves from it every indexed element of its rows of W whose column falls into the
// strip.  The format orders a row's indices by value, then column, so a strip's share of a row is scattered over
// the row's groups: the handle carries a DERIVED strip-major index (built once by cer_prepare_strips from the format
// arrays), whose 16-bit entries hold the rank of the element's value (6 bits: codebooks of at most 64 values) and
// the column inside the strip (10 bits).  The entries of one (strip, row) are padded to a multiple of eight -- a
// chunk of 16 bytes -- with entries of rank 0, whose weight Omega[0] - Omega[0] is zero; the pointers count chunks.
// Every element is multiplied by its own value, so the fragmentation of the groups does not matter.
//
// Lanes: a part of 8 lanes serves one entry at a time (16 bytes = 4 batch columns per lane: one conflict-free LDS
// read of a 128-byte row per entry); all 8 lanes load the same chunk, so the entry reaches them without a
// cross-lane operation, and its weight comes from a table in LDS that is addressed by the entry's top byte (rank and
// the two top column bits; one sub-dword shift forms the address).  kP adjacent parts share one row of W at a time
// (they take its chunks in turn and add their sums at the row's end); a workgroup's rows are dealt to its 128 / kP
// slots in contiguous runs, so a slot walks one contiguous range of chunks, three chunks in flight.  The ends of the
// workgroup's rows are staged in LDS.  Each (strip, row) leaves a partial sum; a second kernel adds the strips'
// partial sums in strip order (deterministic) and the constant term of a non-zero most frequent value (Appendix
// A-A1).
#include "cer_device.hpp"

namespace cer {
namespace {

constexpr uint32_t kStripTile = 32;                               // batch columns per tile: one 128-byte row per entry
constexpr uint32_t kStripBytes = kStripRows * kStripTile * 4u;    // the strip in LDS
constexpr uint32_t kStripWtsBytes = 1024;                         // 256 weights in front of it (LDS address 0)
constexpr uint32_t kStripMaxRows = 4096;                          // rows of W per workgroup (their ends sit in LDS)

typedef float F4 __attribute__((ext_vector_type(4)));
typedef const F4 __attribute__((address_space(3))) * LdsF4Ptr;
typedef const float __attribute__((address_space(3))) * LdsF1Ptr;

// 4 x the byte `kByte` of d: the LDS address of the weight of the entry whose top byte it is.
template <int kByte>
__device__ __forceinline__ uint32_t weight_address(uint32_t d, uint32_t two) {
    uint32_t r;
    if (kByte == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(two), "v"(d));
    else asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(two), "v"(d));
    return r;
}

// One chunk: eight entries, each a 128-byte row of the strip times its weight.  xbase = the lane's 16 bytes inside a
// row + the strip's LDS address.
__device__ __forceinline__ void strip_chunk(const uint4& q, uint32_t xbase, F4& acc) {
    uint32_t two = 2u;
    asm("" : "+v"(two));  // the shift count in a vector register (sub-dword forms take no constants)
    const uint32_t d[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t wa0 = weight_address<1>(d[k], two), wa1 = weight_address<3>(d[k], two);
        uint32_t c0, c1, xa0, xa1;  // written out: one bit-field extract and one shift-add per address
        asm("v_bfe_u32 %0, %1, 0, 10" : "=v"(c0) : "v"(d[k]));
        asm("v_bfe_u32 %0, %1, 16, 10" : "=v"(c1) : "v"(d[k]));
        asm("v_lshl_add_u32 %0, %1, 7, %2" : "=v"(xa0) : "v"(c0), "v"(xbase));
        asm("v_lshl_add_u32 %0, %1, 7, %2" : "=v"(xa1) : "v"(c1), "v"(xbase));
        const float w0 = *reinterpret_cast<LdsF1Ptr>((uintptr_t)wa0);
        const F4 x0 = *reinterpret_cast<LdsF4Ptr>((uintptr_t)xa0);
        const float w1 = *reinterpret_cast<LdsF1Ptr>((uintptr_t)wa1);
        const F4 x1 = *reinterpret_cast<LdsF4Ptr>((uintptr_t)xa1);
        acc.x = fmaf(w0, x0.x, acc.x); acc.y = fmaf(w0, x0.y, acc.y);
        acc.z = fmaf(w0, x0.z, acc.z); acc.w = fmaf(w0, x0.w, acc.w);
        acc.x = fmaf(w1, x1.x, acc.x); acc.y = fmaf(w1, x1.y, acc.y);
        acc.z = fmaf(w1, x1.z, acc.z); acc.w = fmaf(w1, x1.w, acc.w);
    }
}

// chunks: the strip-major index, 16 bytes per chunk, closed by one chunk of zeros (index zero_chunk);
// sptr[s (m + 1) + r] = first chunk of (strip s, row r).
// part: [strip][m][L] partial sums.
template <int kP>
__global__ __launch_bounds__(1024) void cer_strip_kernel(const uint4* __restrict__ chunks, const uint32_t* __restrict__ sptr,
                                                         const float* __restrict__ X, float* __restrict__ part,
                                                         const float* __restrict__ omega, uint32_t m, uint32_t n, uint32_t L,
                                                         uint32_t K, uint32_t ntiles, uint32_t nsplit,
                                                         uint32_t rows_per_split, uint32_t zero_chunk) {
    // LDS: [256 weights][strip: rows of 8 x 16 bytes][ends of the workgroup's rows, in chunks]; no static LDS, so the
    // weight of an entry sits at LDS address 4 x (its top byte).
    extern __shared__ __align__(16) unsigned char strip_smem[];
    float* s_w = reinterpret_cast<float*>(strip_smem);
    F4* xs4 = reinterpret_cast<F4*>(strip_smem + kStripWtsBytes);
    uint32_t* s_end = reinterpret_cast<uint32_t*>(strip_smem + kStripWtsBytes + kStripBytes);
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t split = blockIdx.x % nsplit, tile = (blockIdx.x / nsplit) % ntiles, s = blockIdx.x / (nsplit * ntiles);
    const uint32_t c0 = s * kStripRows, rows_here = min(kStripRows, n - c0);
    const uint32_t r_begin = min(m, split * rows_per_split), rows = min(m, r_begin + rows_per_split) - r_begin;
    const uint32_t* sp = sptr + (size_t)s * (m + 1) + r_begin;

    // the strip of this tile of batch columns: 8 threads copy one 128-byte row, eight loads per thread in flight
    const F4* X4 = reinterpret_cast<const F4*>(X);
    const uint32_t row_f4 = L >> 2;  // 16-byte pieces per row of X
    const uint32_t tile_f4 = min(8u, row_f4 - tile * 8u);  // ... of this tile: fewer than 8 in a ragged last tile
    {
        const uint32_t pieces = rows_here * 8u;
        F4 xr[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t i = min((uint32_t)k * 1024u + threadIdx.x, pieces - 1u);
            // the pieces of the last tile that lie behind the batch's last column re-read the tile's first piece
            xr[k] = X4[(size_t)(c0 + (i >> 3)) * row_f4 + tile * 8u + ((i & 7u) < tile_f4 ? (i & 7u) : 0u)];
        }
        for (uint32_t i = threadIdx.x; i <= rows; i += 1024u) s_end[i] = sp[i];
        if (threadIdx.x < 256u) {
            const uint32_t rank = threadIdx.x >> 2;
            s_w[threadIdx.x] = rank < K ? omega[rank] - omega[0] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t i = (uint32_t)k * 1024u + threadIdx.x;
            if (i < pieces) xs4[i] = xr[k];
        }
    }
    __syncthreads();

    // this lane's slot (kP parts = 8 kP lanes) and its contiguous run of the workgroup's rows
    constexpr uint32_t kSlots = 128u / kP;
    const uint32_t ch = lane & 7u, p = (lane >> 3) & (kP - 1u);
    const uint32_t slot = wave * (8u / kP) + (lane >> 3) / kP;
    const uint32_t ra = slot * rows / kSlots, rb = (slot + 1u) * rows / kSlots;  // rows <= kStripMaxRows: no overflow
    const uint32_t xbase = kStripWtsBytes + ch * 16u;

    // generator: the slot's next chunks; flag bit 0: the slot still has rows, bit 1: its current row ends here.  Free
    // of branches, and every load is issued unconditionally (a part without a chunk of its own reads the chunk of
    // zeros behind the index: entries of rank 0, weight zero), so that the waits for the three chunks in flight stay
    // exact.  gnext = end of the row behind the current one, read from LDS an iteration before it is needed.
    uint32_t gr = ra, gbase = s_end[ra], gce = s_end[min(ra + 1u, rows)], gnext = s_end[min(ra + 2u, rows)];
    auto gen = [&](uint4& q, uint32_t& f) {
        const bool active = gr < rb;
        const bool mine = active && gbase + p < gce;
        q = chunks[mine ? gbase + p : zero_chunk];
        const bool ends = active && gbase + kP >= gce;
        f = (active ? 1u : 0u) | (ends ? 2u : 0u);
        gbase = ends ? gce : (active ? gbase + kP : gbase);
        gce = ends ? gnext : gce;
        gr += ends ? 1u : 0u;
        gnext = s_end[min(gr + 2u, rows)];
    };
    F4 acc = F4{0.f, 0.f, 0.f, 0.f};
    uint32_t cr = ra;  // the row the consumer is in
    F4* out = reinterpret_cast<F4*>(part) + ((size_t)s * m + r_begin) * row_f4 + tile * 8u + ch;
    auto consume = [&](const uint4& q, uint32_t f) {
        strip_chunk(q, xbase, acc);
        if (__ballot((f & 2u) != 0u) != 0ull) {  // some slot of the wave ends a row
            F4 sum = acc;
            if (kP > 1) {
#pragma unroll
                for (uint32_t o = 8u; o < 8u * kP; o <<= 1) {
                    sum.x += __shfl_xor(sum.x, (int)o, kWave); sum.y += __shfl_xor(sum.y, (int)o, kWave);
                    sum.z += __shfl_xor(sum.z, (int)o, kWave); sum.w += __shfl_xor(sum.w, (int)o, kWave);
                }
            }
            if (f & 2u) {
                if (p == 0u && ch < tile_f4) out[(size_t)cr * row_f4] = sum;
                acc = F4{0.f, 0.f, 0.f, 0.f};
                ++cr;
            }
        }
    };
    uint4 qa, qb, qc;
    uint32_t fa, fb, fc;
    gen(qa, fa);
    gen(qb, fb);
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
}

// Y[r][:] = sum over strips of part[s][r][:]  (+ Omega[0] . T[:]), in strip order
__global__ __launch_bounds__(256) void cer_strip_sum_kernel(const float* __restrict__ part, float* __restrict__ Y,
                                                            const float* __restrict__ T, float omega0, uint32_t nstrips,
                                                            uint64_t plane_f4, uint32_t row_f4) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= plane_f4) return;
    const F4* p = reinterpret_cast<const F4*>(part);
    F4 a = p[i];
    for (uint32_t s = 1; s < nstrips; ++s) {
        const F4 b = p[(uint64_t)s * plane_f4 + i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    if (omega0 != 0.f) {
        const F4 t = reinterpret_cast<const F4*>(T)[i % row_f4];
        a.x = fmaf(omega0, t.x, a.x); a.y = fmaf(omega0, t.y, a.y);
        a.z = fmaf(omega0, t.z, a.z); a.w = fmaf(omega0, t.w, a.w);
    }
    reinterpret_cast<F4*>(Y)[i] = a;
}

constexpr size_t strip_lds_bytes(uint32_t rows) { return (size_t)kStripWtsBytes + kStripBytes + 4u * ((size_t)rows + 1u); }

}  // namespace

bool strip_applicable(const DeviceView& d, const float* X, const float* Y, uint32_t L) {
    return d.strip_idx != nullptr && d.n_strips > 0 && L >= kStripTile && L % 4u == 0 && d.m > 0 &&
           (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15u) == 0 &&
           d.lds_per_block >= strip_lds_bytes(kStripMaxRows) + 512;
}

// Launch shape of the strip kernel for a batch of L columns, and a rough duration.
//   * One workgroup per compute unit holds 128 KB of LDS, so the (strip, tile) pairs are split over the rows into
//     about as many workgroups as there are compute units (never more than kStripMaxRows rows each).
//   * Parts per row: enough rows for every slot (four or more each), but no more parts than a (strip, row) has
//     chunks to keep them busy.
//   * Duration (measured on MI355X: AlexNet-fc6 shape batch 32 / 64 / 128: 30 / 46 / 78 us, VGG-fc6 shape batch 32 /
//     64 / 128: 38 / 52 / 92 us, 3x3 convolution shape batch 3136: 268 us): a slot's rows x its chunk rounds per row,
//     0.62 us per round with 16 waves on a compute unit (vector ALU and LDS both close to busy: 83 vector
//     instructions and 17 LDS reads per 64 entries), per round of workgroups; 6 us for the launch, the staging of
//     the strip and the tail; the second kernel reads strips x m x L partial sums.
StripPlan plan_strip(const DeviceView& d, uint32_t L, int parts) {
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
    p.P = 1;
    while (p.P < 8 && p.rows_per_split * p.P < 4u * 128u && chunks_per_row >= 4.0 * p.P) p.P *= 2;
    if (parts == 1 || parts == 2 || parts == 4 || parts == 8) p.P = (uint32_t)parts;
    const double rows_per_slot = std::ceil((double)p.rows_per_split * p.P / 128.0);
    const double rounds = rows_per_slot * (chunks_per_row / p.P + (p.P - 1) / (2.0 * p.P));
    const double wg_rounds = std::ceil((double)p.blocks / std::max(d.cus, 1));
    const double partial_bytes = (double)d.n_strips * m * L * 4.0;
    p.est_us = wg_rounds * (rounds * 0.62 + 3.0) + 3.0 + (3.0 + 2.0 * partial_bytes / 5e6);
    return p;
}

hipError_t launch_strip(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream,
                        const MatmulOptions& o) {
    const uint32_t m = (uint32_t)d.m, n = (uint32_t)d.n;
    const StripPlan sp = plan_strip(d, L, o.strip_parts);
    const uint32_t ntiles = sp.ntiles, nsplit = sp.nsplit, rows_per_split = sp.rows_per_split, P = sp.P;
    const uint64_t blocks = sp.blocks;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    float* part = nullptr;
    const size_t part_bytes = (size_t)d.n_strips * m * L * sizeof(float);
    hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&part), part_bytes, stream);
    if (e != hipSuccess) return e;
    const size_t lds = strip_lds_bytes(rows_per_split);
    static LdsGrant<4> grant;
    const void* kernels[4] = {reinterpret_cast<const void*>(cer_strip_kernel<1>), reinterpret_cast<const void*>(cer_strip_kernel<2>),
                              reinterpret_cast<const void*>(cer_strip_kernel<4>), reinterpret_cast<const void*>(cer_strip_kernel<8>)};
    const int slot = P == 1 ? 0 : (P == 2 ? 1 : (P == 4 ? 2 : 3));
    e = grant.ensure(slot, kernels[slot], strip_lds_bytes(kStripMaxRows));
    if (e == hipSuccess) {
#define CER_STRIP_LAUNCH(PP)                                                                                           \
    hipLaunchKernelGGL(cer_strip_kernel<PP>, dim3((uint32_t)blocks), dim3(1024), lds, stream,                          \
                       static_cast<const uint4*>(d.strip_idx), d.strip_ptr, X, part, d.omega, m, n, L, (uint32_t)d.K,  \
                       ntiles, nsplit, rows_per_split, (uint32_t)d.strip_chunks)
        switch (P) {
            case 1: CER_STRIP_LAUNCH(1); break;
            case 2: CER_STRIP_LAUNCH(2); break;
            case 4: CER_STRIP_LAUNCH(4); break;
            default: CER_STRIP_LAUNCH(8); break;
        }
#undef CER_STRIP_LAUNCH
        e = hipGetLastError();
    }
    if (e == hipSuccess) {
        const uint64_t plane_f4 = (uint64_t)m * (L / 4);
        hipLaunchKernelGGL(cer_strip_sum_kernel, dim3((uint32_t)((plane_f4 + 255) / 256)), dim3(256), 0, stream, part, Y, T,
                           d.omega0, d.n_strips, plane_f4, L / 4);
        e = hipGetLastError();
    }
    const hipError_t f = (hipError_t)temp_free(part, stream);
    return e == hipSuccess ? f : e;
}

}  // namespace cer
