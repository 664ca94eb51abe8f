// Batch 1 (one input vector): Y = W.x with W in CER / CSER form (Appendix A-C, Algorithms 3 and 4 of the paper; the
// constant term of a non-zero most frequent value, Appendix A-A1, is summed from the staged copy of x).
//
// X is staged into LDS once per workgroup and gathered from there; one wave per row, lane l of step s owns the
// row's (64 s + l)-th index; the 64 lane totals are combined with DPP cross-lane adds.  Two kernels: the cursor
// kernel keeps the paper's order of operations (sum a group's inputs, multiply once), the expansion kernel serves
// rows of many short groups.
#include "cer_device.hpp"

namespace cer {
namespace {

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
// Launch logic
// ------------------------------------------------------------------------------------------------

// LDS the batch-1 kernels may claim dynamically: the device's limit less its few static words.
size_t gemv_lds_budget(const DeviceView& d) { return d.lds_per_block - 256; }

// Whether the cursor kernel stages X in LDS for this matrix: whenever it fits beside Omega and the group lists of
// 4 waves (with at least 64 entries each).
bool gemv_stages_x(const DeviceView& d, const MatmulOptions& o) {
    const size_t x_bytes = (((size_t)d.n + 3) & ~(size_t)3) * sizeof(float);
    const size_t om_bytes = d.K <= 4096 ? (((size_t)d.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    const uint32_t gcap = std::max<uint32_t>(1u, (uint32_t)std::min<int64_t>(d.max_row_groups, 1022));
    return (o.flags & kOptXFromGlobal) == 0 &&
           x_bytes + om_bytes + (size_t)4 * (std::min<uint32_t>(gcap, 64u) + 2) * 8 <= gemv_lds_budget(d);
}

template <typename IdxT>
hipError_t launch_gemv(const DeviceView& d, const KView& k, const float* X, float* Y, const float* T, hipStream_t stream,
                       const MatmulOptions& o) {
    const size_t budget = gemv_lds_budget(d);
    const size_t x_bytes = (((size_t)k.n + 3) & ~(size_t)3) * sizeof(float);
    const bool omega_in_lds = k.K <= 4096;
    const size_t om_bytes = omega_in_lds ? (((size_t)k.K + 3) & ~(size_t)3) * sizeof(float) : 0;
    // per-wave list of non-empty groups: as long as the longest row needs, at most 1022 entries
    uint32_t gcap = std::max<uint32_t>(1u, (uint32_t)std::min<int64_t>(d.max_row_groups, 1022));
    auto list_bytes = [&](int waves) { return (size_t)waves * (gcap + 2) * 8; };
    const bool x_in_lds = gemv_stages_x(d, o);
    const size_t fixed = (x_in_lds ? x_bytes : 0) + om_bytes;
    // a workgroup that stages a large X should own many rows: 16 waves; small X: 4 waves, more workgroups
    int waves = (x_in_lds && x_bytes > 40 * 1024) ? 16 : 4;
    while (fixed + list_bytes(waves) > budget && waves > 4) waves >>= 1;
    while (fixed + list_bytes(waves) > budget && gcap > 64) gcap = std::max<uint32_t>(64u, gcap / 2);
    const size_t lds = fixed + list_bytes(waves);
    if (lds > budget) return hipErrorInvalidValue;
    // resident workgroups per CU, limited by LDS and by 32 waves per CU
    size_t per_cu = std::min<size_t>(d.lds_per_block / (lds + 256), (size_t)(32 / waves));
    per_cu = std::max<size_t>(1, std::min<size_t>(per_cu, 8));
    const uint64_t slots = (uint64_t)d.cus * per_cu;
    const uint32_t iters = std::max<uint32_t>((uint32_t)((k.m + slots * waves - 1) / (slots * waves)), 1u);
    const uint32_t rows_per_block = iters * waves;
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
    if (lds > 48 * 1024) {
        static LdsGrant<3 * 18> grant;  // per index width
        const int kslot = (x_in_lds ? (vec4 ? 2 : 1) : 0) + (k.cser ? 3 : 0) + (few ? 6 : 0) + (one ? 6 : 0);
        const int wslot = sizeof(IdxT) == 1 ? 0 : (sizeof(IdxT) == 2 ? 1 : 2);
        const hipError_t e = grant.ensure(wslot * 18 + kslot, reinterpret_cast<const void*>(kern), budget);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, stream, k, X, Y, T, rows_per_block,
                       omega_in_lds ? 1 : 0, gcap);
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

// The expansion kernel's plan for this matrix if the product would use it (waves == 0 otherwise): preferred by the
// caller (whenever X fits in LDS), ruled out by a preference for the cursor kernel, else for rows of short groups.
GemvExpandPlan gemv_expand_choice(const DeviceView& d, const MatmulOptions& o) {
    if (o.path == 4 || (o.path != 0 && gemv_expand_pays(d))) return plan_gemv_expand(d);
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
