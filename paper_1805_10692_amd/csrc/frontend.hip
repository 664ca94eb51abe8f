// Device front-end: a dense fp32 weight matrix that already lives in HBM goes to CER / CSER without a
// trip through the host -- optionally through the uniform quantizer of Section V-B first.
//
//   range     min / max of W (quantizer only); the K = 2^b points of the codebook
//   codes     element -> codebook position (quantizer: nearest point; otherwise: exact look-up),
//             one byte per element, and a per-row histogram over the positions
//   rank      global histogram -> frequency-major order Omega (Section II-A, step 1)
//   layout    per row: number of indexed elements and of groups; exclusive scans over the rows give
//             every row its slice of colI and of OmegaPtr / OmegaI
//   emit      per row: a stable counting sort of the columns by rank writes colI, the bucket ends are
//             the row's pointers (steps 2-4)
//
// One wave owns one row in `layout` and `emit`, so no two waves ever write the same output element
// and the result does not depend on scheduling: it is the same array, bit for bit, as the host
// encoder's.  Codebooks of up to 256 values are supported here (one byte per code).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "../../include/cer.h"
#include "cer_internal.hpp"

namespace {

constexpr int kWave = 64;
constexpr int kCodes = 256;  // most codebook positions a byte can name

enum : uint32_t {
    kFlagNonFinite = 1u,  // NaN or infinity among the weights
    kFlagMissing = 2u,    // element that is no codebook value
    kFlagCollide = 4u,    // range too narrow: two of the 2^b points coincide
    kFlagTooLarge = 8u,   // 32-bit offsets do not reach
};

// Small block of device memory the kernels communicate through; copied to the host once.
struct FrontState {
    float wmin, wmax, step;
    uint32_t flags;
    uint32_t K;         // codebook positions in use (caller's K, or the quantizer's point count)
    uint32_t Kp;        // values that occur = length of Omega
    uint32_t max_row_groups;
    uint32_t pad_;
    unsigned long long nnz, G, nonempty;
    unsigned long long hist[kCodes];   // occurrences by codebook position
    unsigned long long count[kCodes];  // occurrences by rank
    float codebook[kCodes];            // value by codebook position
    float sorted_val[kCodes];          // look-up path: codebook sorted by value ...
    uint32_t sorted_pos[kCodes];       // ... and the position each came from
    float omega[kCodes];               // value by rank
    uint32_t rank_of[kCodes];          // codebook position -> rank
    uint32_t pos_of[kCodes];           // rank -> codebook position
};

__device__ __forceinline__ uint32_t lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// LDS traffic of one wave is ordered; this only keeps the compiler from moving accesses across.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float canonical(float v) { return v == 0.0f ? 0.0f : v; }

// ------------------------------------------------------------------------------------------------
// range: min / max / finiteness
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void range_kernel(const float* __restrict__ W, int64_t N, float* __restrict__ part_min,
                                                    float* __restrict__ part_max, uint32_t* __restrict__ part_bad) {
    float lo = INFINITY, hi = -INFINITY;
    uint32_t bad = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const float w = W[i];
        bad |= (uint32_t)!(fabsf(w) <= 3.402823466e+38f);
        lo = fminf(lo, w);
        hi = fmaxf(hi, w);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
        bad |= (uint32_t)__shfl_xor((int)bad, off, kWave);
    }
    __shared__ float s_lo[4], s_hi[4];
    __shared__ uint32_t s_bad[4];
    const uint32_t wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63u) == 0) {
        s_lo[wave] = lo;
        s_hi[wave] = hi;
        s_bad[wave] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        part_min[blockIdx.x] = fminf(fminf(s_lo[0], s_lo[1]), fminf(s_lo[2], s_lo[3]));
        part_max[blockIdx.x] = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
        part_bad[blockIdx.x] = s_bad[0] | s_bad[1] | s_bad[2] | s_bad[3];
    }
}

// One block of 256 threads: finish the reduction, then lay the K = 2^bits points on the range
// (Section V-B).  Every operation rounds once, to binary32: step = (max - min) / (K - 1),
// point_j = min + j.step, the last point is max itself.  A constant matrix has one point.
__global__ __launch_bounds__(256) void points_kernel(const float* __restrict__ part_min, const float* __restrict__ part_max,
                                                     const uint32_t* __restrict__ part_bad, int nparts, int bits,
                                                     FrontState* __restrict__ st) {
#pragma clang fp contract(off)
    __shared__ float s_lo[256], s_hi[256];
    __shared__ uint32_t s_bad[256];
    __shared__ float s_pts[kCodes];
    const uint32_t t = threadIdx.x;
    float lo = INFINITY, hi = -INFINITY;
    uint32_t bad = 0;
    for (int i = (int)t; i < nparts; i += 256) {
        lo = fminf(lo, part_min[i]);
        hi = fmaxf(hi, part_max[i]);
        bad |= part_bad[i];
    }
    s_lo[t] = lo;
    s_hi[t] = hi;
    s_bad[t] = bad;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)t < off) {
            s_lo[t] = fminf(s_lo[t], s_lo[t + off]);
            s_hi[t] = fmaxf(s_hi[t], s_hi[t + off]);
            s_bad[t] |= s_bad[t + off];
        }
        __syncthreads();
    }
    const float wmin = s_lo[0] + 0.0f, wmax = s_hi[0] + 0.0f;  // -0.0 -> +0.0
    const uint32_t K = (wmin == wmax) ? 1u : (1u << bits);
    const float step = (K > 1) ? (wmax - wmin) / (float)(K - 1) : 0.0f;
    float p = 0.f;
    if (t < K) {
        const float prod = (float)t * step;
        p = prod + wmin;
        if (t == K - 1) p = wmax;
        if (K == 1) p = wmin;
        st->codebook[t] = p;
    }
    s_pts[t] = p;
    __syncthreads();
    uint32_t flags = s_bad[0] ? kFlagNonFinite : 0u;
    if (t + 1 < K && !(s_pts[t + 1] > s_pts[t])) atomicOr(&st->flags, kFlagCollide);
    if (t == 0) {
        st->wmin = wmin;
        st->wmax = wmax;
        st->step = step;
        st->K = K;
        if (flags) atomicOr(&st->flags, flags);
    }
}

// ------------------------------------------------------------------------------------------------
// codes: element -> codebook position; per-row histogram.  One workgroup per row (a flat array is
// cut into rows of row_len elements).
// ------------------------------------------------------------------------------------------------
template <bool kQuant>
__global__ __launch_bounds__(256) void codes_kernel(const float* __restrict__ W, int64_t total, int64_t row_len,
                                                    FrontState* __restrict__ st, uint8_t* __restrict__ codes,
                                                    uint32_t* __restrict__ cnt, float* __restrict__ Wq) {
#pragma clang fp contract(off)
    __shared__ uint32_t s_hist[kCodes];
    __shared__ float s_val[kCodes];
    __shared__ uint32_t s_pos[kCodes];
    const uint32_t t = threadIdx.x;
    const int64_t r = blockIdx.x;
    const uint32_t K = st->K;
    s_hist[t] = 0;
    if (kQuant) {
        s_val[t] = t < K ? st->codebook[t] : 0.f;
    } else {
        s_val[t] = t < K ? st->sorted_val[t] : 0.f;
        s_pos[t] = t < K ? st->sorted_pos[t] : 0u;
    }
    __syncthreads();
    const float wmin = st->wmin, step = st->step, top = (float)(K - 1);
    const float* row = W + r * row_len;
    uint8_t* crow = codes ? codes + r * row_len : nullptr;
    const int64_t n = min(row_len, total - r * row_len);  // the last row of a flat array may be short
    bool missing = false;
    for (int64_t j0 = 0; j0 < n; j0 += 256) {
        const int64_t j = j0 + t;
        const bool in = j < n;
        uint32_t code = 0;
        if (in) {
            const float w = row[j];
            if (kQuant) {
                // nearest point, decided in binary32: round-half-even of the scaled coordinate
                float q = 0.f;
                if (K > 1) {
                    const float d = w - wmin;
                    q = fminf(fmaxf(rintf(d / step), 0.f), top);
                }
                code = (uint32_t)q;
                if (Wq) Wq[r * row_len + j] = s_val[code];
            } else {
                const float c = canonical(w);
                uint32_t lo = 0, hi = K;  // first sorted value that is not below c
                while (lo < hi) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (s_val[mid] < c) lo = mid + 1; else hi = mid;
                }
                const bool hit = lo < K && __float_as_uint(s_val[lo]) == __float_as_uint(c);
                missing |= !hit;
                code = hit ? s_pos[lo] : 0u;
            }
            if (crow) crow[j] = (uint8_t)code;
        }
        // histogram: the lanes that share the first active lane's code are counted with one add
        const uint64_t act = __ballot(in);
        if (act) {
            const uint32_t lead = (uint32_t)__builtin_amdgcn_readfirstlane((int)code);
            const uint64_t same = __ballot(in && code == lead);
            if (in && code != lead) atomicAdd(&s_hist[code], 1u);
            if ((uint64_t)__builtin_ctzll(act) == (uint64_t)(t & 63u)) atomicAdd(&s_hist[lead], (uint32_t)__popcll(same));
        }
    }
    if (__syncthreads_or(missing) && t == 0) atomicOr(&st->flags, kFlagMissing);
    cnt[r * kCodes + t] = s_hist[t];
}

// Global histogram = column sums of the per-row histograms.
__global__ __launch_bounds__(256) void hist_kernel(const uint32_t* __restrict__ cnt, int64_t m, int64_t rows_per_block,
                                                   FrontState* __restrict__ st) {
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block, r1 = min(m, r0 + rows_per_block);
    unsigned long long s = 0;
    for (int64_t r = r0; r < r1; ++r) s += cnt[r * kCodes + threadIdx.x];
    if (s) atomicAdd(&st->hist[threadIdx.x], s);
}

// Frequency-major order: higher count first, equal counts in codebook order; values that never
// occur are left out (Section II-A, step 1).  One block of 256 threads, K <= 256: each thread
// finds its own position by counting who comes before it.
__global__ __launch_bounds__(256) void rank_kernel(FrontState* __restrict__ st) {
    __shared__ unsigned long long s_h[kCodes];
    const uint32_t t = threadIdx.x, K = st->K;
    const unsigned long long c = t < K ? st->hist[t] : 0ull;
    s_h[t] = c;
    __syncthreads();
    uint32_t before = 0, occurring = 0;
    for (uint32_t j = 0; j < K; ++j) {
        const unsigned long long cj = s_h[j];
        occurring += cj > 0;
        before += (cj > c) || (cj == c && j < t);
    }
    st->rank_of[t] = c > 0 ? before : 0u;
    if (c > 0) {
        st->pos_of[before] = t;
        st->omega[before] = canonical(st->codebook[t]);
        st->count[before] = c;
    }
    if (t == 0) st->Kp = occurring;
}

// ------------------------------------------------------------------------------------------------
// layout: per row, the number of indexed elements and of groups.  One wave per row.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_layout_kernel(const uint32_t* __restrict__ cnt, int64_t m, int cser,
                                                         FrontState* __restrict__ st, uint32_t* __restrict__ rowG,
                                                         uint32_t* __restrict__ rowN) {
    const uint32_t lane = threadIdx.x & 63u;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= m) return;
    uint32_t present = 0, topk = 0, nn = 0;
#pragma unroll
    for (int i = 0; i < kCodes / kWave; ++i) {
        const uint32_t pos = lane + 64u * i;
        const uint32_t c = cnt[r * kCodes + pos];
        const uint32_t k = st->rank_of[pos];
        if (c > 0 && k >= 1) {
            ++present;
            topk = max(topk, k);
            nn += c;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        present += __shfl_xor(present, off, kWave);
        nn += __shfl_xor(nn, off, kWave);
        topk = max(topk, (uint32_t)__shfl_xor((int)topk, off, kWave));
    }
    if (lane == 0) {
        const uint32_t g = cser ? present : topk;  // CER keeps the empty groups below the row's highest rank
        rowG[r] = g;
        rowN[r] = nn;
        if (present) atomicAdd(&st->nonempty, (unsigned long long)present);
        atomicMax(&st->max_row_groups, g);
    }
}

// Exclusive prefix sums of rowG and rowN over the rows, m + 1 entries each.  One block.
__global__ __launch_bounds__(1024) void scan_rows_kernel(const uint32_t* __restrict__ rowG, const uint32_t* __restrict__ rowN,
                                                         int64_t m, uint32_t* __restrict__ rowPtr, uint32_t* __restrict__ rowOff,
                                                         FrontState* __restrict__ st) {
    __shared__ unsigned long long s_g[16], s_n[16];
    __shared__ unsigned long long s_carry[2];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    if (t == 0) s_carry[0] = s_carry[1] = 0;
    __syncthreads();
    for (int64_t base = 0; base < m; base += 1024) {
        const int64_t r = base + t;
        const unsigned long long g = r < m ? rowG[r] : 0u, nn = r < m ? rowN[r] : 0u;
        unsigned long long ig = g, in_ = nn;  // inclusive scans inside the wave
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const unsigned long long ug = __shfl_up(ig, off, kWave), un = __shfl_up(in_, off, kWave);
            if ((int)lane >= off) {
                ig += ug;
                in_ += un;
            }
        }
        if (lane == 63) {
            s_g[wave] = ig;
            s_n[wave] = in_;
        }
        __syncthreads();
        unsigned long long og = s_carry[0], on = s_carry[1];
        for (uint32_t w = 0; w < wave; ++w) {
            og += s_g[w];
            on += s_n[w];
        }
        if (r < m) {
            rowPtr[r] = (uint32_t)(og + ig - g);
            rowOff[r] = (uint32_t)(on + in_ - nn);
        }
        __syncthreads();
        if (t == 1023) {
            s_carry[0] = og + ig;
            s_carry[1] = on + in_;
        }
        __syncthreads();
    }
    if (t == 0) {
        const unsigned long long G = s_carry[0], nnz = s_carry[1];
        st->G = G;
        st->nnz = nnz;
        rowPtr[m] = (uint32_t)G;
        rowOff[m] = (uint32_t)nnz;
        // the product kernels address colI and OmegaPtr with 32-bit offsets and read ahead of a row's end
        const unsigned long long limit = 0xFFFFFFFFull - 65536;
        if (G > limit || nnz > limit) atomicOr(&st->flags, kFlagTooLarge);
    }
}

// ------------------------------------------------------------------------------------------------
// emit: the row's pointers and its columns, grouped by rank.  One wave per row.
// ------------------------------------------------------------------------------------------------
template <typename ColT, typename OiT>
__global__ __launch_bounds__(256) void emit_kernel(const uint8_t* __restrict__ codes, const uint32_t* __restrict__ cnt,
                                                   const uint32_t* __restrict__ rowPtrTmp, const uint32_t* __restrict__ rowOffTmp,
                                                   const FrontState* __restrict__ st, int64_t m, int64_t n, int cser,
                                                   ColT* __restrict__ colI, uint32_t* __restrict__ omegaPtr,
                                                   uint32_t* __restrict__ rowPtr, uint2* __restrict__ rowInfo,
                                                   OiT* __restrict__ omegaI) {
    __shared__ uint32_t s_rank[kCodes];
    __shared__ uint32_t s_fill[4][kCodes];  // next free colI slot of each rank's bucket
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    s_rank[threadIdx.x] = st->rank_of[threadIdx.x];
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 4 + wave;
    if (r >= m) return;
    uint32_t* fill = s_fill[wave];
    const uint32_t Kp = st->Kp;
    const uint32_t g0 = rowPtrTmp[r], off0 = rowOffTmp[r];
    const uint32_t groups = rowPtrTmp[r + 1] - g0;
    if (lane == 0) {
        rowPtr[r] = g0;
        rowInfo[r] = make_uint2(g0, off0);
        if (r == 0) omegaPtr[0] = 0;
        if (r == m - 1) {
            rowPtr[m] = rowPtrTmp[m];
            rowInfo[m] = make_uint2(rowPtrTmp[m], rowOffTmp[m]);
        }
    }
    // bucket sizes by rank -> bucket starts (exclusive scan over ranks 1, 2, ...) and the pointers
    uint32_t carry = 0, gcarry = 0;
#pragma unroll
    for (int i = 0; i < kCodes / kWave; ++i) {
        const uint32_t k = lane + 64u * i;
        const uint32_t c = (k >= 1 && k < Kp) ? cnt[r * kCodes + st->pos_of[k]] : 0u;
        uint32_t inc = c;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t u = __shfl_up(inc, off, kWave);
            if ((int)lane >= off) inc += u;
        }
        const uint32_t end = off0 + carry + inc;
        fill[k] = end - c;
        const uint64_t pres = __ballot(c > 0);
        if (cser) {
            if (c > 0) {
                const uint32_t idx = gcarry + (uint32_t)__popcll(pres & ((1ull << lane) - 1ull));
                omegaPtr[g0 + idx + 1] = end;
                omegaI[g0 + idx] = (OiT)k;
            }
            gcarry += (uint32_t)__popcll(pres);
        } else if (k >= 1 && k <= groups) {
            omegaPtr[g0 + k] = end;  // an empty group repeats the previous pointer
        }
        carry += (uint32_t)__shfl((int)inc, 63, kWave);
    }
    wave_lds_sync();
    // stable scatter: 64 consecutive columns at a time; lanes with the same rank are found with one
    // ballot per bit of the rank and take consecutive slots in lane (= column) order
    const uint32_t nbits = 32u - (uint32_t)__builtin_clz(Kp > 1 ? Kp - 1 : 1u);
    const uint64_t below = (1ull << lane) - 1ull;
    const uint8_t* crow = codes + r * n;
    for (int64_t j0 = 0; j0 < n; j0 += kWave) {
        const int64_t j = j0 + lane;
        const uint32_t k = j < n ? s_rank[crow[j]] : 0u;
        const bool act = k >= 1;
        uint64_t peers = __ballot(act);
        if (!peers) continue;
        for (uint32_t b = 0; b < nbits; ++b) {
            const bool bit = (k >> b) & 1u;
            const uint64_t votes = __ballot(bit);
            peers &= bit ? votes : ~votes;
        }
        if (act) {
            const uint32_t before = (uint32_t)__popcll(peers & below);
            const uint32_t slot = fill[k];
            colI[slot + before] = (ColT)j;
            if (before == 0) fill[k] = slot + (uint32_t)__popcll(peers);
        }
        wave_lds_sync();
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct DeviceBuf {
    void* p = nullptr;
    ~DeviceBuf() {
        if (p) (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1); }
    template <typename T>
    T* as() const {
        return static_cast<T*>(p);
    }
};

void narrow_u32(const std::vector<uint32_t>& src, int bits, cer::HostArray* dst) {
    dst->len = (int64_t)src.size();
    dst->bits = bits;
    dst->bytes.resize(src.size() * (size_t)(bits / 8));
    if (bits == 8) {
        for (size_t i = 0; i < src.size(); ++i) dst->bytes[i] = (uint8_t)src[i];
    } else if (bits == 16) {
        auto* p = reinterpret_cast<uint16_t*>(dst->bytes.data());
        for (size_t i = 0; i < src.size(); ++i) p[i] = (uint16_t)src[i];
    } else if (!src.empty()) {
        std::memcpy(dst->bytes.data(), src.data(), src.size() * 4);
    }
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        const hipError_t e_ = (expr);                   \
        if (e_ != hipSuccess) return cer::record_hip_error((int)e_); \
    } while (0)

// Runs range/points (bits > 0) or takes the caller's codebook, then codes + per-row histograms over
// `rows` rows of row_len elements (the last one possibly shorter).  Returns after the stream has drained.
int run_codes(const float* W, int64_t total, int64_t rows, int64_t row_len, const float* codebook, int32_t K, int32_t bits,
              hipStream_t s, FrontState* st_dev, uint8_t* codes, uint32_t* cnt, float* Wq) {
    FrontState init;
    std::memset(&init, 0, sizeof init);
    DeviceBuf part;
    if (bits > 0) {
        const int nparts = (int)std::min<int64_t>(2048, (total + 255) / 256);
        HIP_TRY(part.alloc((size_t)nparts * 12));
        float* pmin = part.as<float>();
        float* pmax = pmin + nparts;
        uint32_t* pbad = reinterpret_cast<uint32_t*>(pmax + nparts);
        HIP_TRY(hipMemcpyAsync(st_dev, &init, sizeof init, hipMemcpyHostToDevice, s));
        range_kernel<<<nparts, 256, 0, s>>>(W, total, pmin, pmax, pbad);
        points_kernel<<<1, 256, 0, s>>>(pmin, pmax, pbad, nparts, bits, st_dev);
        codes_kernel<true><<<(unsigned)rows, 256, 0, s>>>(W, total, row_len, st_dev, codes, cnt, Wq);
    } else {
        // codebook sorted by value for the look-up; duplicates and non-finite values are refused
        std::vector<uint32_t> order((size_t)K);
        for (int32_t k = 0; k < K; ++k) {
            if (!std::isfinite(codebook[k])) return CER_E_BAD_CODEBOOK;
            order[(size_t)k] = (uint32_t)k;
            init.codebook[k] = codebook[k] == 0.0f ? 0.0f : codebook[k];
        }
        std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return init.codebook[a] < init.codebook[b]; });
        for (int32_t k = 0; k < K; ++k) {
            init.sorted_val[k] = init.codebook[order[(size_t)k]];
            init.sorted_pos[k] = order[(size_t)k];
            if (k > 0 && init.sorted_val[k] == init.sorted_val[k - 1]) return CER_E_BAD_CODEBOOK;
        }
        init.K = (uint32_t)K;
        HIP_TRY(hipMemcpyAsync(st_dev, &init, sizeof init, hipMemcpyHostToDevice, s));
        codes_kernel<false><<<(unsigned)rows, 256, 0, s>>>(W, total, row_len, st_dev, codes, cnt, nullptr);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));  // `part` and `init` must outlive the work queued on them
    return CER_OK;
}

int flags_to_error(uint32_t flags) {
    if (flags & kFlagNonFinite) return CER_E_INVALID;
    if (flags & kFlagMissing) return CER_E_NOT_IN_CODEBOOK;
    if (flags & kFlagCollide) return CER_E_BAD_CODEBOOK;
    if (flags & kFlagTooLarge) return CER_E_TOO_LARGE;
    return CER_OK;
}

template <typename ColT>
void launch_emit(int oi_bits, unsigned blocks, hipStream_t s, const uint8_t* codes, const uint32_t* cnt,
                 const uint32_t* rowPtrTmp, const uint32_t* rowOffTmp, const FrontState* st, int64_t m, int64_t n, int cser,
                 unsigned char* b, const cer::DeviceLayout& l) {
    auto* colI = reinterpret_cast<ColT*>(b + l.off_colI);
    auto* optr = reinterpret_cast<uint32_t*>(b + l.off_optr);
    auto* rptr = reinterpret_cast<uint32_t*>(b + l.off_rptr);
    auto* info = reinterpret_cast<uint2*>(b + l.off_ri);
    // rank < K <= 256, so OmegaI is always one byte wide here
    (void)oi_bits;
    emit_kernel<ColT, uint8_t><<<blocks, 256, 0, s>>>(codes, cnt, rowPtrTmp, rowOffTmp, st, m, n, cser, colI, optr, rptr, info,
                                                      reinterpret_cast<uint8_t*>(b + l.off_oi));
}

}  // namespace

namespace cer {

int quantize_device(const float* W, int64_t count, int32_t bits, uint8_t* codes, float* Wq, float* codebook_out,
                    int32_t* K_out, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t row_len = 4096, rows = (count + row_len - 1) / row_len;
    DeviceBuf st, cnt;
    HIP_TRY(st.alloc(sizeof(FrontState)));
    HIP_TRY(cnt.alloc((size_t)rows * kCodes * 4));
    int rc = run_codes(W, count, rows, row_len, nullptr, 0, bits, s, st.as<FrontState>(), codes, cnt.as<uint32_t>(), Wq);
    if (rc != CER_OK) return rc;
    FrontState h;
    HIP_TRY(hipMemcpy(&h, st.p, sizeof h, hipMemcpyDeviceToHost));
    rc = flags_to_error(h.flags);
    if (rc != CER_OK) return rc;
    if (K_out) *K_out = (int32_t)h.K;
    if (codebook_out) std::memcpy(codebook_out, h.codebook, (size_t)h.K * 4);
    return CER_OK;
}

int encode_device(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, int32_t bits, bool cser,
                  void* stream, float* codebook_out, int32_t* K_out, cer_matrix** out) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t N = m * n;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));

    DeviceBuf st, codes, cnt, rowG, rowN, rowPtrTmp, rowOffTmp;
    HIP_TRY(st.alloc(sizeof(FrontState)));
    HIP_TRY(codes.alloc((size_t)N));
    HIP_TRY(cnt.alloc((size_t)m * kCodes * 4));
    HIP_TRY(rowG.alloc((size_t)m * 4));
    HIP_TRY(rowN.alloc((size_t)m * 4));
    HIP_TRY(rowPtrTmp.alloc((size_t)(m + 1) * 4));
    HIP_TRY(rowOffTmp.alloc((size_t)(m + 1) * 4));
    FrontState* sd = st.as<FrontState>();

    int rc = run_codes(W, N, m, n, codebook, K, bits, s, sd, codes.as<uint8_t>(), cnt.as<uint32_t>(), nullptr);
    if (rc != CER_OK) return rc;
    const unsigned row_blocks = (unsigned)((m + 3) / 4);
    const int64_t rows_per_block = 64;
    hist_kernel<<<(unsigned)((m + rows_per_block - 1) / rows_per_block), 256, 0, s>>>(cnt.as<uint32_t>(), m, rows_per_block, sd);
    rank_kernel<<<1, 256, 0, s>>>(sd);
    row_layout_kernel<<<row_blocks, 256, 0, s>>>(cnt.as<uint32_t>(), m, cser ? 1 : 0, sd, rowG.as<uint32_t>(), rowN.as<uint32_t>());
    scan_rows_kernel<<<1, 1024, 0, s>>>(rowG.as<uint32_t>(), rowN.as<uint32_t>(), m, rowPtrTmp.as<uint32_t>(),
                                        rowOffTmp.as<uint32_t>(), sd);
    HIP_TRY(hipGetLastError());
    FrontState h;
    HIP_TRY(hipMemcpyAsync(&h, sd, sizeof h, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    rc = flags_to_error(h.flags);
    if (rc != CER_OK) return rc;
    if (K_out) *K_out = (int32_t)h.K;
    if (codebook_out) std::memcpy(codebook_out, h.codebook, (size_t)h.K * 4);

    // sizes are known: the handle's allocation, filled in place
    auto A = std::make_shared<HostMatrix>();
    A->cser = cser;
    A->m = m;
    A->n = n;
    A->K = (int32_t)h.Kp;
    A->nnz = (int64_t)h.nnz;
    A->G = (int64_t)h.G;
    A->nonempty_groups = (int64_t)h.nonempty;
    A->max_row_groups = (int64_t)h.max_row_groups;
    A->omega.assign(h.omega, h.omega + h.Kp);
    A->count.assign(h.count, h.count + h.Kp);
    const int col_bits = min_index_bits(n > 0 ? (uint64_t)(n - 1) : 0);
    const int oi_bits = min_index_bits(A->K > 0 ? (uint64_t)(A->K - 1) : 0);
    const size_t colI_bytes = (size_t)A->nnz * (size_t)(col_bits / 8);
    const size_t oi_bytes = cser ? (size_t)A->G * (size_t)(oi_bits / 8) : 0;
    const DeviceLayout l = DeviceLayout::make(colI_bytes, A->G, m, oi_bytes, A->K);
    DeviceBuf base;
    HIP_TRY(base.alloc(l.total));
    auto* b = base.as<unsigned char>();
    HIP_TRY(hipMemsetAsync(b, 0, l.total, s));
    HIP_TRY(hipMemcpyAsync(b + l.off_om, h.omega, (size_t)h.Kp * 4, hipMemcpyHostToDevice, s));
    switch (col_bits) {
        case 8:
            launch_emit<uint8_t>(oi_bits, row_blocks, s, codes.as<uint8_t>(), cnt.as<uint32_t>(), rowPtrTmp.as<uint32_t>(),
                                 rowOffTmp.as<uint32_t>(), sd, m, n, cser ? 1 : 0, b, l);
            break;
        case 16:
            launch_emit<uint16_t>(oi_bits, row_blocks, s, codes.as<uint8_t>(), cnt.as<uint32_t>(), rowPtrTmp.as<uint32_t>(),
                                  rowOffTmp.as<uint32_t>(), sd, m, n, cser ? 1 : 0, b, l);
            break;
        default:
            launch_emit<uint32_t>(oi_bits, row_blocks, s, codes.as<uint8_t>(), cnt.as<uint32_t>(), rowPtrTmp.as<uint32_t>(),
                                  rowOffTmp.as<uint32_t>(), sd, m, n, cser ? 1 : 0, b, l);
    }
    HIP_TRY(hipGetLastError());

    // host mirror of the arrays (inspection, decode, clones), pointer arrays at their minimal widths
    std::vector<uint32_t> optr((size_t)A->G + 1), rptr((size_t)m + 1);
    A->colI.len = A->nnz;
    A->colI.bits = col_bits;
    A->colI.bytes.resize(colI_bytes);
    if (colI_bytes) HIP_TRY(hipMemcpyAsync(A->colI.bytes.data(), b + l.off_colI, colI_bytes, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(optr.data(), b + l.off_optr, optr.size() * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(rptr.data(), b + l.off_rptr, rptr.size() * 4, hipMemcpyDeviceToHost, s));
    if (cser) {
        A->omegaI.len = A->G;
        A->omegaI.bits = oi_bits;
        A->omegaI.bytes.resize(oi_bytes);
        if (oi_bytes) HIP_TRY(hipMemcpyAsync(A->omegaI.bytes.data(), b + l.off_oi, oi_bytes, hipMemcpyDeviceToHost, s));
    }
    HIP_TRY(hipStreamSynchronize(s));
    narrow_u32(optr, min_index_bits((uint64_t)A->nnz), &A->omegaPtr);
    narrow_u32(rptr, min_index_bits((uint64_t)A->G), &A->rowPtr);

    auto* hnd = new cer_matrix();
    hnd->host = std::move(A);
    bind_device(hnd, dev, base.p, l);
    base.p = nullptr;  // now owned by the handle
    *out = hnd;
    return CER_OK;
}

}  // namespace cer
