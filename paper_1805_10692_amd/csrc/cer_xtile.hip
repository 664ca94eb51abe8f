// Batch > 1 with a narrow tile of X resident in LDS: the reuse of input elements that Section V-C of the paper
// names as the missing optimisation.
#include "cer_device.hpp"

namespace cer {
namespace {

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
// Launch logic
// ------------------------------------------------------------------------------------------------

template <typename IdxT, int V, int U>
hipError_t launch_xtile_v(const DeviceView& d, const KView& k, const XtilePlan& p, const float* Xp, uint32_t raw_x, float* Y,
                          const float* T, uint32_t L, hipStream_t stream, int slot) {
    using Kern = void (*)(KView, const float*, float*, const float*, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t);
    Kern kern = k.cser ? cer_xtile_kernel<IdxT, V, U, true> : cer_xtile_kernel<IdxT, V, U, false>;
    if (p.lds > 48 * 1024) {
        static LdsGrant<12> grant;
        const hipError_t e = grant.ensure(slot * 2 + (k.cser ? 1 : 0), reinterpret_cast<const void*>(kern), d.lds_per_block);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(kXtWaves * kWave), p.lds, stream, k, Xp, Y, T, L, p.ntiles, p.rpw, p.pcap,
                       raw_x);
    return hipGetLastError();
}

template <typename IdxT>
hipError_t launch_xtile(const DeviceView& d, const KView& k, const XtilePlan& p, const float* X, float* Y, const float* T,
                        uint32_t L, hipStream_t stream, int idx_slot) {
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
    hipError_t e = p.V == 8 ? launch_xtile_v<IdxT, 8, 3>(d, k, p, Xp, raw_x, Y, T, L, stream, idx_slot * 2 + 1)
                            : launch_xtile_v<IdxT, 4, 8>(d, k, p, Xp, raw_x, Y, T, L, stream, idx_slot * 2);
    if (tmp) {
        hipError_t f = (hipError_t)temp_free(tmp, stream);
        if (e == hipSuccess) e = f;
    }
    return e;
}

}  // namespace

XtilePlan plan_xtile(const DeviceView& d, uint32_t L) {
    XtilePlan p;
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
            if (lds > d.lds_per_block) break;
            const uint64_t rowblocks = ((uint64_t)d.m + (uint64_t)kXtWaves * rpw - 1) / ((uint64_t)kXtWaves * rpw);
            const uint64_t blocks = rowblocks * ntiles;
            if (blocks > 0x7FFFFFFFull) continue;
            const double rounds = (double)((blocks + d.cus - 1) / d.cus);
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

hipError_t launch_xtile_any(const DeviceView& d, const XtilePlan& p, const float* X, float* Y, const float* T, uint32_t L,
                            hipStream_t stream) {
    const KView k = make_kview(d);
    switch (d.colI_bits) {
        case 8: return launch_xtile<uint8_t>(d, k, p, X, Y, T, L, stream, 0);
        case 16: return launch_xtile<uint16_t>(d, k, p, X, Y, T, L, stream, 1);
        default: return launch_xtile<uint32_t>(d, k, p, X, Y, T, L, stream, 2);
    }
}

}  // namespace cer
