// Device front-end: a dense fp32 weight matrix that already lives in HBM goes to CER / CSER without a
// trip through the host -- optionally through the uniform quantizer of Section V-B first.
//
//   range     min / max of W (quantizer only); the K = 2^b points of the codebook
//   codes     element -> codebook position (quantizer: nearest point; otherwise: exact look-up),
//             one byte per element, and a per-row histogram over the positions
//   rank      global histogram -> frequency-major order Omega (Section III-A, step 1)
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
#include <mutex>
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
    uint32_t max_row_nnz;  // indexed elements of the longest row
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
__device__ __forceinline__ void range_take(float w, float& lo, float& hi, uint32_t& bad) {
    bad |= (uint32_t)!(fabsf(w) <= 3.402823466e+38f);
    lo = fminf(lo, w);
    hi = fmaxf(hi, w);
}

__global__ __launch_bounds__(256) void range_kernel(const float* __restrict__ W, int64_t N, float* __restrict__ part_min,
                                                    float* __restrict__ part_max, uint32_t* __restrict__ part_bad) {
    float lo = INFINITY, hi = -INFINITY;
    uint32_t bad = 0;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
    // the bulk in 16-byte pieces (W is aligned by the caller's allocator or the scalar loop below takes it all)
    const int64_t N4 = ((reinterpret_cast<uintptr_t>(W) & 15u) == 0) ? N / 4 : 0;
    const float4* W4 = reinterpret_cast<const float4*>(W);
    for (int64_t i = tid; i < N4; i += stride) {
        const float4 w = W4[i];
        range_take(w.x, lo, hi, bad);
        range_take(w.y, lo, hi, bad);
        range_take(w.z, lo, hi, bad);
        range_take(w.w, lo, hi, bad);
    }
    for (int64_t i = N4 * 4 + tid; i < N; i += stride) range_take(W[i], lo, hi, bad);
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
    if (t + 1 < K && !(s_pts[t + 1] > s_pts[t])) atomicOr(&st->flags, kFlagCollide);
    if (t == 0) {
        st->wmin = wmin;
        st->wmax = wmax;
        st->step = step;
        st->K = K;
        if (s_bad[0]) atomicOr(&st->flags, kFlagNonFinite);
    }
}

// ------------------------------------------------------------------------------------------------
// codes: element -> codebook position; per-row histogram.  One workgroup per row (a flat array is
// cut into rows of row_len elements).
// ------------------------------------------------------------------------------------------------
// Look-up of a value's codebook position: open-addressing hash table in LDS over the bit patterns of the (at most
// 256) codebook values; a free slot holds a pattern no finite value has.
constexpr uint32_t kHashSlots = 1024, kHashFree = 0xFFFFFFFFu;
__device__ __forceinline__ uint32_t hash_slot(uint32_t bits) { return (bits * 2654435761u) >> 22; }

struct CodeCtx {
    uint32_t K;
    float wmin, step, top;
    const float* val;      // LDS: quantizer -> points by position
    const uint32_t* hkey;  // LDS: look-up -> bit pattern stored in each hash slot
    const uint32_t* hpos;  // LDS: look-up -> codebook position of that value
};

template <bool kQuant>
__device__ __forceinline__ uint32_t code_of(float w, const CodeCtx& c, bool& missing) {
#pragma clang fp contract(off)
    if (kQuant) {
        // nearest point, decided in binary32: round-half-even of the scaled coordinate
        float q = 0.f;
        if (c.K > 1) {
            const float d = w - c.wmin;
            q = fminf(fmaxf(rintf(d / c.step), 0.f), c.top);
        }
        return (uint32_t)q;
    }
    const uint32_t bits = __float_as_uint(canonical(w));
    uint32_t h = hash_slot(bits);
    for (;;) {
        const uint32_t key = c.hkey[h];
        if (key == kHashFree) {  // not a codebook value (the table always has free slots)
            missing = true;
            return 0u;
        }
        if (key == bits) return c.hpos[h];
        h = (h + 1u) & (kHashSlots - 1u);
    }
}

// Each thread takes four consecutive elements per round: one 16-byte load, four codes, one 4-byte
// store (a row whose length or address does not allow that falls back to single elements).
template <bool kQuant>
__global__ __launch_bounds__(256) void codes_kernel(const float* __restrict__ W, int64_t total, int64_t row_len,
                                                    FrontState* __restrict__ st, uint8_t* __restrict__ codes,
                                                    uint32_t* __restrict__ cnt, float* __restrict__ Wq, int vec_ok) {
    __shared__ uint32_t s_hist[kCodes];
    __shared__ float s_val[kCodes];
    __shared__ uint32_t s_hkey[kQuant ? 1 : kHashSlots], s_hpos[kQuant ? 1 : kHashSlots];
    const uint32_t t = threadIdx.x;
    const int64_t r = blockIdx.x;
    CodeCtx c;
    c.K = st->K;
    s_hist[t] = 0;
    if (kQuant) {
        s_val[t] = t < c.K ? st->codebook[t] : 0.f;
    } else {
        for (uint32_t i = t; i < kHashSlots; i += 256) s_hkey[i] = kHashFree;
        __syncthreads();
        if (t < c.K) {
            const uint32_t bits = __float_as_uint(canonical(st->sorted_val[t]));
            uint32_t h = hash_slot(bits);
            while (atomicCAS(&s_hkey[h], kHashFree, bits) != kHashFree) h = (h + 1u) & (kHashSlots - 1u);
            s_hpos[h] = st->sorted_pos[t];
        }
    }
    __syncthreads();
    c.wmin = st->wmin;
    c.step = st->step;
    c.top = (float)(c.K - 1);
    c.val = s_val;
    c.hkey = s_hkey;
    c.hpos = s_hpos;
    const float* row = W + r * row_len;
    uint8_t* crow = codes ? codes + r * row_len : nullptr;
    float* qrow = Wq ? Wq + r * row_len : nullptr;
    const int64_t n = min(row_len, total - r * row_len);  // the last row of a flat array may be short
    bool missing = false;
    // the next round's four elements are requested before this round's are coded
    float4 ahead = make_float4(0.f, 0.f, 0.f, 0.f);
    if (vec_ok && 4 * (int64_t)t + 4 <= n) ahead = *reinterpret_cast<const float4*>(row + 4 * (int64_t)t);
    for (int64_t j0 = 0; j0 < n; j0 += 1024) {
        const int64_t j = j0 + 4 * (int64_t)t;
        uint32_t code[4] = {0, 0, 0, 0};
        const int valid = (int)max((int64_t)0, min((int64_t)4, n - j));
        const float4 w = ahead;
        if (vec_ok && j + 1024 + 4 <= n) ahead = *reinterpret_cast<const float4*>(row + j + 1024);
        if (valid == 4 && vec_ok) {
            code[0] = code_of<kQuant>(w.x, c, missing);
            code[1] = code_of<kQuant>(w.y, c, missing);
            code[2] = code_of<kQuant>(w.z, c, missing);
            code[3] = code_of<kQuant>(w.w, c, missing);
            if (crow) *reinterpret_cast<uint32_t*>(crow + j) = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
            if (kQuant && qrow)
                *reinterpret_cast<float4*>(qrow + j) = make_float4(s_val[code[0]], s_val[code[1]], s_val[code[2]], s_val[code[3]]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (e < valid) {
                    code[e] = code_of<kQuant>(row[j + e], c, missing);
                    if (crow) crow[j + e] = (uint8_t)code[e];
                    if (kQuant && qrow) qrow[j + e] = s_val[code[e]];
                }
            }
        }
        // histogram: everything that equals the first active lane's first code is counted with one add
        const uint64_t act = __ballot(valid > 0);
        if (act) {
            const uint32_t lead = (uint32_t)__builtin_amdgcn_readfirstlane((int)code[0]);
            uint32_t same = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool in = e < valid;
                same += (uint32_t)__popcll(__ballot(in && code[e] == lead));
                if (in && code[e] != lead) atomicAdd(&s_hist[code[e]], 1u);
            }
            if ((uint32_t)__builtin_ctzll(act) == (t & 63u)) atomicAdd(&s_hist[lead], same);
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
// occur are left out (Section III-A, step 1).  One block of 256 threads, K <= 256: each thread
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
// layout: per row, the number of indexed elements, of groups and of non-empty groups.  One wave per row.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void row_layout_kernel(const uint32_t* __restrict__ cnt, int64_t m, int cser,
                                                         const FrontState* __restrict__ st, uint32_t* __restrict__ rowG,
                                                         uint32_t* __restrict__ rowN, uint32_t* __restrict__ rowP) {
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
        rowG[r] = cser ? present : topk;  // CER keeps the empty groups below the row's highest rank
        rowN[r] = nn;
        rowP[r] = present;
    }
}

// Exclusive prefix sums of rowG and rowN over the rows (m + 1 entries each), the number of
// non-empty groups and the largest group count of a row.  One block.
__global__ __launch_bounds__(1024) void scan_rows_kernel(const uint32_t* __restrict__ rowG, const uint32_t* __restrict__ rowN,
                                                         const uint32_t* __restrict__ rowP, int64_t m,
                                                         uint32_t* __restrict__ rowPtr, uint32_t* __restrict__ rowOff,
                                                         FrontState* __restrict__ st) {
    __shared__ unsigned long long s_g[16], s_n[16], s_p[16];
    __shared__ uint32_t s_mx[16], s_ml[16];
    __shared__ unsigned long long s_carry[2];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    if (t == 0) s_carry[0] = s_carry[1] = 0;
    unsigned long long my_p = 0;
    uint32_t my_mx = 0, my_ml = 0;
    __syncthreads();
    for (int64_t base = 0; base < m; base += 1024) {
        const int64_t r = base + t;
        const unsigned long long g = r < m ? rowG[r] : 0u, nn = r < m ? rowN[r] : 0u;
        my_p += r < m ? rowP[r] : 0u;
        my_mx = max(my_mx, (uint32_t)g);
        my_ml = max(my_ml, (uint32_t)nn);
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
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        my_p += __shfl_xor(my_p, off, kWave);
        my_mx = max(my_mx, (uint32_t)__shfl_xor((int)my_mx, off, kWave));
        my_ml = max(my_ml, (uint32_t)__shfl_xor((int)my_ml, off, kWave));
    }
    if (lane == 0) {
        s_p[wave] = my_p;
        s_mx[wave] = my_mx;
        s_ml[wave] = my_ml;
    }
    __syncthreads();
    if (t == 0) {
        unsigned long long p = 0;
        uint32_t mx = 0, ml = 0;
        for (int w = 0; w < 16; ++w) {
            p += s_p[w];
            mx = max(mx, s_mx[w]);
            ml = max(ml, s_ml[w]);
        }
        st->max_row_nnz = ml;
        const unsigned long long G = s_carry[0], nnz = s_carry[1];
        st->G = G;
        st->nnz = nnz;
        st->nonempty = p;
        st->max_row_groups = mx;
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
// 64 consecutive columns: lanes with the same rank are found with one ballot per bit of the rank
// and take consecutive slots of that rank's bucket in lane (= column) order.
template <typename ColT>
__device__ __forceinline__ void scatter64(uint32_t k, int64_t j, uint32_t nbits, uint64_t below, uint32_t* fill,
                                          unsigned long long* marks, ColT* __restrict__ colI) {
    const bool act = k >= 1;
    uint64_t peers = __ballot(act);
    if (!peers) return;
    if (nbits > 3) {
        // many ranks: the lanes of a rank meet in that rank's 64-bit word in LDS (all words are zero between calls)
        if (act) atomicOr(&marks[k], below + 1ull);  // below = 2^lane - 1
        wave_lds_sync();
        if (act) peers = marks[k];
    } else {
        for (uint32_t b = 0; b < nbits; ++b) {
            const bool bit = (k >> b) & 1u;
            const uint64_t votes = __ballot(bit);
            peers &= bit ? votes : ~votes;
        }
    }
    if (act) {
        const uint32_t before = (uint32_t)__popcll(peers & below);
        const uint32_t slot = fill[k];
        colI[slot + before] = (ColT)j;
        if (before == 0) {
            fill[k] = slot + (uint32_t)__popcll(peers);
            if (nbits > 3) marks[k] = 0ull;
        }
    }
    wave_lds_sync();
}

constexpr uint32_t kEmitStage = 1024;  // staged entries per wave

template <typename ColT, typename OiT>
__global__ __launch_bounds__(256) void emit_kernel(const uint8_t* __restrict__ codes, const uint32_t* __restrict__ cnt,
                                                   const uint32_t* __restrict__ rowPtrTmp, const uint32_t* __restrict__ rowOffTmp,
                                                   const FrontState* __restrict__ st, int64_t m, int64_t n, int cser,
                                                   int sparse, ColT* __restrict__ colI, uint32_t* __restrict__ omegaPtr,
                                                   uint32_t* __restrict__ rowPtr, uint2* __restrict__ rowInfo,
                                                   OiT* __restrict__ omegaI) {
    __shared__ uint32_t s_rank[kCodes];
    __shared__ uint32_t s_fill[4][kCodes];  // next free colI slot of each rank's bucket
    __shared__ uint32_t s_stage[4][kEmitStage];  // (column << 8) | rank of the columns waiting for the scatter
    __shared__ unsigned long long s_marks[4][kCodes];  // per rank: the lanes of the current batch that hold it
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    s_rank[threadIdx.x] = st->rank_of[threadIdx.x];
#pragma unroll
    for (int w = 0; w < 4; ++w) s_marks[w][threadIdx.x] = 0ull;
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 4 + wave;
    if (r >= m) return;
    uint32_t* fill = s_fill[wave];
    unsigned long long* marks = s_marks[wave];
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
    // stable scatter of the row's columns into the buckets
    const uint32_t nbits = 32u - (uint32_t)__builtin_clz(Kp > 1 ? Kp - 1 : 1u);
    const uint64_t below = (1ull << lane) - 1ull;
    const uint8_t* crow = codes + r * n;
    if (sparse && (n & 3) == 0 && (reinterpret_cast<uintptr_t>(codes) & 3u) == 0 && n <= (int64_t)1 << 24) {
        // 256 columns per round: each lane loads the codes of four consecutive columns at once (the
        // next round's are requested before this round's are used).  Most columns hold the most
        // frequent value and take no part in the scatter: the others are first packed, in column order,
        // as (column, rank) into a buffer in LDS -- four ballots per 256 columns -- and the scatter with
        // its ballot per rank bit then runs over full batches of 64 buffered entries.
        uint32_t* buf = s_stage[wave];
        uint32_t held = 0;  // wave-uniform
        auto drain = [&](uint32_t keep_below) {
            // scatters buffered entries in batches of 64 until fewer than keep_below remain
            uint32_t done = 0;
            while (held - done >= keep_below && held > done) {
                const uint32_t i = done + lane;
                const uint32_t e = i < held ? buf[i] : 0u;
                scatter64<ColT>(e & 0xFFu, (int64_t)(e >> 8), nbits, below, fill, marks, colI);
                done += kWave;
            }
            if (done >= held) {
                held = 0;
            } else {
                // fewer than 64 left: move them to the front
                const uint32_t rest = held - done;
                const uint32_t e = lane < rest ? buf[done + lane] : 0u;
                wave_lds_sync();
                if (lane < rest) buf[lane] = e;
                wave_lds_sync();
                held = rest;
            }
        };
        const uint32_t* crow4 = reinterpret_cast<const uint32_t*>(crow);
        const int64_t n4 = n >> 2;
        // the code words of four rounds are in flight: a round is short against the memory latency
        constexpr int kAhead = 4;
        uint32_t ring[kAhead];
#pragma unroll
        for (int d = 0; d < kAhead; ++d) ring[d] = 64 * d + lane < n4 ? crow4[64 * d + lane] : 0u;
        for (int64_t jb = 0; jb < n; jb += 256 * kAhead) {
#pragma unroll
            for (int d = 0; d < kAhead; ++d) {
                const int64_t j0 = jb + 256 * d;  // may lie beyond the row: then no lane is inside
                const uint32_t cur = ring[d];
                const int64_t q = ((j0 + 256 * kAhead) >> 2) + lane;
                ring[d] = q < n4 ? crow4[q] : 0u;
                // this lane's four columns are consecutive, so lane order is column order
                const uint32_t c0 = (uint32_t)j0 + 4u * lane;
                const bool inside = j0 + 4 * (int64_t)lane < n;
                uint32_t k[4];
                uint32_t pos = held, total = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    k[i] = inside ? s_rank[(cur >> (8 * i)) & 0xFFu] : 0u;
                    const uint64_t some = __ballot(k[i] >= 1);
                    pos += (uint32_t)__popcll(some & below);
                    total += (uint32_t)__popcll(some);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (k[i] >= 1) buf[pos++] = ((c0 + (uint32_t)i) << 8) | k[i];
                }
                held += total;
                if (held > kEmitStage - 256) {
                    wave_lds_sync();
                    drain(kWave);
                }
            }
        }
        wave_lds_sync();
        drain(1);
    } else if ((n & 3) == 0 && (reinterpret_cast<uintptr_t>(codes) & 3u) == 0) {
        // as above without the buffer (most columns take part): a shuffle hands every lane the code of its own
        // column, 64 consecutive columns per scatter
        const uint32_t* crow4 = reinterpret_cast<const uint32_t*>(crow);
        const int64_t n4 = n >> 2;
        constexpr int kAhead = 4;
        uint32_t ring[kAhead];
#pragma unroll
        for (int d = 0; d < kAhead; ++d) ring[d] = 64 * d + lane < n4 ? crow4[64 * d + lane] : 0u;
        for (int64_t jb = 0; jb < n; jb += 256 * kAhead) {
#pragma unroll
            for (int d = 0; d < kAhead; ++d) {
                const int64_t j0 = jb + 256 * d;
                const uint32_t cur = ring[d];
                const int64_t q = ((j0 + 256 * kAhead) >> 2) + lane;
                ring[d] = q < n4 ? crow4[q] : 0u;
                if (j0 >= n) break;  // uniform
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int64_t j = j0 + 64 * s + lane;
                    const uint32_t v = (uint32_t)__shfl((int)cur, 16 * s + (int)(lane >> 2), kWave);
                    const uint32_t code = (v >> (8u * (lane & 3u))) & 0xFFu;
                    scatter64<ColT>(j < n ? s_rank[code] : 0u, j, nbits, below, fill, marks, colI);
                }
            }
        }
    } else {
        for (int64_t j0 = 0; j0 < n; j0 += kWave) {
            const int64_t j = j0 + lane;
            scatter64<ColT>(j < n ? s_rank[crow[j]] : 0u, j, nbits, below, fill, marks, colI);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// decode: format arrays -> dense matrix (Section III-A: M is reconstructed uniquely).  One workgroup
// per row (large matrices) or per (row, every gridDim.y-th segment).  A segment of up to kDecSeg
// columns is assembled in LDS -- filled with Omega[0], then every indexed position of the row whose
// column falls into the segment writes its group's value -- and written out once with 16-byte stores,
// so that HBM sees every line of W exactly once.  Positions are spread over the threads, kDecPer per
// thread with all index loads issued together; a position finds its group by a binary search in the
// row's pointers (up to kDecThreads groups at a time in LDS; repeated pointers, CER's empty groups,
// are skipped by the search).  A row of at most kDecThreads groups and kDecThreads.kDecPer positions
// keeps its columns and values in registers for all its segments; a larger row reloads them per
// segment.
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kDecSeg = 4096;

// kDecThreads = workgroup size: 256, or 64 for matrices of short rows (a row is then little work, and four times as
// many workgroups are in flight).  kDecPer = positions a thread keeps in registers: 8 for sparse rows, 32 where rows
// hold thousands of indices.
template <typename ColT, uint32_t kDecThreads, uint32_t kDecPer>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(
    const ColT* __restrict__ colI, const uint32_t* __restrict__ omegaPtr, const uint32_t* __restrict__ rowPtr,
    const uint8_t* __restrict__ omegaI, int oi_bits, const float* __restrict__ omega, int cser, int64_t n,
    uint32_t seg, uint32_t nseg, float* __restrict__ W) {
    extern __shared__ __align__(16) float s_row[];  // seg floats
    __shared__ uint32_t s_ptr[kDecThreads + 1];
    __shared__ float s_val[kDecThreads];
    constexpr uint32_t T = kDecThreads, P = kDecPer;
    const uint32_t tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    const float w0 = omega[0];
    const uint32_t g0 = rowPtr[r], g1 = rowPtr[r + 1];

    // pointers and values of the groups gb .. gb + cnt - 1 of this row -> LDS
    auto stage_groups = [&](uint32_t gb, uint32_t cnt) {
        if (tid < cnt) {
            const uint32_t g = gb + tid;
            uint32_t rank = g - g0 + 1u;  // Algorithm 3: position in the row; Algorithm 4: OmegaI
            if (cser) {
                rank = oi_bits == 8 ? omegaI[g]
                                    : (oi_bits == 16 ? reinterpret_cast<const uint16_t*>(omegaI)[g]
                                                     : reinterpret_cast<const uint32_t*>(omegaI)[g]);
            }
            s_ptr[tid] = omegaPtr[g];
            s_val[tid] = omega[rank];
        }
        if (tid == 0) s_ptr[cnt] = omegaPtr[gb + cnt];
    };
    // columns and values of the positions pb + tid + k.T < pe (k < P) of the staged groups -> registers
    uint32_t col[P];
    float val[P];
    uint32_t ok = 0;
    auto load_positions = [&](uint32_t pb, uint32_t pe, uint32_t cnt) {
        ok = 0;
        const uint32_t last = pe > pb ? pe - 1u : pb;  // loads behind the last position are redirected to it
#pragma unroll
        for (uint32_t k = 0; k < P; ++k) col[k] = (uint32_t)colI[min(pb + tid + k * T, last)];
        uint32_t lo = 0;  // a thread's positions grow with k, and so do their groups: the search resumes where it was
#pragma unroll
        for (uint32_t k = 0; k < P; ++k) {
            const uint32_t p = pb + tid + k * T;
            val[k] = 0.f;
            if (p < pe) {
                if (s_ptr[lo + 1u] <= p) {  // not the same group as the previous position
                    uint32_t hi = cnt;      // s_ptr[lo] <= p < s_ptr[hi]
                    while (hi - lo > 1u) {
                        const uint32_t mid = (lo + hi) >> 1;
                        if (s_ptr[mid] <= p) lo = mid; else hi = mid;
                    }
                }
                val[k] = s_val[lo];
                ok |= 1u << k;
            }
        }
    };
    auto scatter = [&](int64_t c0, uint32_t len) {
#pragma unroll
        for (uint32_t k = 0; k < P; ++k) {
            const uint64_t rel = (uint64_t)col[k] - (uint64_t)c0;  // huge when left of the segment
            if (((ok >> k) & 1u) && rel < len) s_row[rel] = val[k];
        }
    };

    const uint32_t ngroups = g1 - g0;
    bool resident = ngroups <= T;
    if (resident && ngroups > 0) {
        stage_groups(g0, ngroups);
        __syncthreads();
        const uint32_t pb = s_ptr[0], pe = s_ptr[ngroups];
        resident = pe - pb <= T * P;  // uniform over the workgroup
        if (resident) load_positions(pb, pe, ngroups);
    }

    for (uint32_t si = blockIdx.y; si < nseg; si += gridDim.y) {  // uniform over the workgroup
        const int64_t c0 = (int64_t)si * seg;
        if (c0 >= n) break;
        const uint32_t len = (uint32_t)((n - c0) < (int64_t)seg ? (n - c0) : (int64_t)seg);  // 1 .. seg
        {
            const float4 f4 = make_float4(w0, w0, w0, w0);
            const uint32_t n4 = (len + 3u) >> 2;
            for (uint32_t j = tid; j < n4; j += T) reinterpret_cast<float4*>(s_row)[j] = f4;
        }
        __syncthreads();
        if (resident) {
            scatter(c0, len);
        } else {
            for (uint32_t gb = g0; gb < g1; gb += T) {
                const uint32_t cnt = g1 - gb < T ? g1 - gb : T;
                __syncthreads();  // nobody still searches the previous groups
                stage_groups(gb, cnt);
                __syncthreads();
                const uint32_t pe = s_ptr[cnt];
                for (uint32_t pb = s_ptr[0]; pb < pe; pb += T * P) {
                    load_positions(pb, pe, cnt);
                    scatter(c0, len);
                }
            }
        }
        __syncthreads();
        float* out = W + r * n + c0;
        if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
            const uint32_t n4 = len >> 2;
            for (uint32_t j = tid; j < n4; j += T) reinterpret_cast<float4*>(out)[j] = reinterpret_cast<const float4*>(s_row)[j];
            for (uint32_t j = (n4 << 2) + tid; j < len; j += T) out[j] = s_row[j];
        } else {
            for (uint32_t j = tid; j < len; j += T) out[j] = s_row[j];
        }
        __syncthreads();  // the segment has been read before the next one is filled
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
// Temporary device memory from the stream-ordered pool: released when the work queued before the
// release has run, so the buffers can be dropped as soon as the last kernel using them is queued.
struct DeviceBuf {
    void* p = nullptr;
    hipStream_t s = nullptr;
    ~DeviceBuf() {
        if (p) (void)cer::temp_free(p, s);
    }
    hipError_t alloc(size_t bytes, hipStream_t stream) {
        s = stream;
        return (hipError_t)cer::temp_alloc(&p, bytes ? bytes : 1, stream);
    }
    template <typename T>
    T* as() const {
        return static_cast<T*>(p);
    }
};

#define HIP_TRY(expr)                                                \
    do {                                                             \
        const hipError_t e_ = (expr);                                \
        if (e_ != hipSuccess) return cer::record_hip_error((int)e_); \
    } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Runs range/points (bits > 0) or takes the caller's codebook, then codes + per-row histograms over
// `rows` rows of row_len elements (the last one possibly shorter).  Returns after the stream has drained.
int run_codes(const float* W, int64_t total, int64_t rows, int64_t row_len, const float* codebook, int32_t K, int32_t bits,
              hipStream_t s, FrontState* st_dev, uint8_t* codes, uint32_t* cnt, float* Wq) {
    FrontState init;
    std::memset(&init, 0, sizeof init);
    const int vec_ok = (row_len % 4 == 0 && aligned16(W) && (!Wq || aligned16(Wq)) &&
                        (!codes || (reinterpret_cast<uintptr_t>(codes) & 3u) == 0)) ? 1 : 0;
    DeviceBuf part;
    if (bits > 0) {
        const int nparts = (int)std::min<int64_t>(2048, (total + 1023) / 1024);
        HIP_TRY(part.alloc((size_t)nparts * 12, s));
        float* pmin = part.as<float>();
        float* pmax = pmin + nparts;
        uint32_t* pbad = reinterpret_cast<uint32_t*>(pmax + nparts);
        HIP_TRY(hipMemcpyAsync(st_dev, &init, sizeof init, hipMemcpyHostToDevice, s));
        range_kernel<<<nparts, 256, 0, s>>>(W, total, pmin, pmax, pbad);
        points_kernel<<<1, 256, 0, s>>>(pmin, pmax, pbad, nparts, bits, st_dev);
        codes_kernel<true><<<(unsigned)rows, 256, 0, s>>>(W, total, row_len, st_dev, codes, cnt, Wq, vec_ok);
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
        codes_kernel<false><<<(unsigned)rows, 256, 0, s>>>(W, total, row_len, st_dev, codes, cnt, nullptr, vec_ok);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(s));  // `init` lives on this frame
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
void launch_emit(unsigned blocks, hipStream_t s, const uint8_t* codes, const uint32_t* cnt, const uint32_t* rowPtrTmp,
                 const uint32_t* rowOffTmp, const FrontState* st, int64_t m, int64_t n, int cser, int sparse,
                 unsigned char* b, const cer::DeviceLayout& l) {
    // rank < K <= 256, so OmegaI is always one byte wide here
    emit_kernel<ColT, uint8_t><<<blocks, 256, 0, s>>>(
        codes, cnt, rowPtrTmp, rowOffTmp, st, m, n, cser, sparse, reinterpret_cast<ColT*>(b + l.off_colI),
        reinterpret_cast<uint32_t*>(b + l.off_optr), reinterpret_cast<uint32_t*>(b + l.off_rptr),
        reinterpret_cast<uint2*>(b + l.off_ri), reinterpret_cast<uint8_t*>(b + l.off_oi));
}

}  // namespace

namespace cer {

namespace {
template <typename ColT>
int launch_decode(const DeviceView& v, float* W, hipStream_t s) {
    // segments of equal length (a multiple of 4 columns, so that aligned rows give aligned segments)
    const int64_t nseg = (v.n + kDecSeg - 1) / kDecSeg;
    const uint32_t seg = (uint32_t)((((v.n + nseg - 1) / nseg) + 3) & ~(int64_t)3);
    if (v.m > 0x7FFFFFFFll || nseg > 0x7FFFFFFFll) return CER_E_INVALID;
    // one workgroup per row walks all its segments, unless that gives too few workgroups to fill the chip
    const int64_t split = std::min<int64_t>(std::min<int64_t>(nseg, 65535), std::max<int64_t>(1, 4096 / v.m));
    const dim3 grid((unsigned)v.m, (unsigned)split);
    const size_t lds = (size_t)seg * sizeof(float);
    if (v.nnz > v.m * 1500)  // rows of thousands of indices: keep up to 8192 of them in registers over the row's segments
        decode_kernel<ColT, 256, 32><<<grid, 256, lds, s>>>(
            static_cast<const ColT*>(v.colI), v.omegaPtr, v.rowPtr, static_cast<const uint8_t*>(v.omegaI), v.omegaI_bits,
            v.omega, v.cser, v.n, seg, (uint32_t)nseg, W);
    else if (v.n <= 1024)  // short rows: one wave per row
        decode_kernel<ColT, 64, 8><<<grid, 64, lds, s>>>(
            static_cast<const ColT*>(v.colI), v.omegaPtr, v.rowPtr, static_cast<const uint8_t*>(v.omegaI), v.omegaI_bits,
            v.omega, v.cser, v.n, seg, (uint32_t)nseg, W);
    else
        decode_kernel<ColT, 256, 8><<<grid, 256, lds, s>>>(
            static_cast<const ColT*>(v.colI), v.omegaPtr, v.rowPtr, static_cast<const uint8_t*>(v.omegaI), v.omegaI_bits,
            v.omega, v.cser, v.n, seg, (uint32_t)nseg, W);
    HIP_TRY(hipGetLastError());
    return CER_OK;
}
}  // namespace

int decode_device(const DeviceView& v, float* W, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (v.m == 0 || v.n == 0) return CER_OK;
    switch (v.colI_bits) {
        case 8: return launch_decode<uint8_t>(v, W, s);
        case 16: return launch_decode<uint16_t>(v, W, s);
        default: return launch_decode<uint32_t>(v, W, s);
    }
}

int quantize_device(const float* W, int64_t count, int32_t bits, uint8_t* codes, float* Wq, float* codebook_out,
                    int32_t* K_out, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t row_len = 4096, rows = (count + row_len - 1) / row_len;
    DeviceBuf st, cnt;
    HIP_TRY(st.alloc(sizeof(FrontState), s));
    HIP_TRY(cnt.alloc((size_t)rows * kCodes * 4, s));
    int rc = run_codes(W, count, rows, row_len, nullptr, 0, bits, s, st.as<FrontState>(), codes, cnt.as<uint32_t>(), Wq);
    if (rc != CER_OK) return rc;
    FrontState h;
    HIP_TRY(hipMemcpyAsync(&h, st.p, sizeof h, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
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

    // one stream-ordered temporary: [state][codes: N bytes][per-row histograms][rowG, rowN, rowP [m], rowPtrTmp, rowOffTmp [m + 1]]
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t off_codes = up(sizeof(FrontState)), off_cnt = off_codes + up((size_t)N);
    const size_t off_rows = off_cnt + up((size_t)m * kCodes * 4), tmp_bytes = off_rows + up((size_t)(5 * m + 2) * 4);
    DeviceBuf tmp;
    HIP_TRY(tmp.alloc(tmp_bytes, s));
    unsigned char* tp = tmp.as<unsigned char>();
    FrontState* sd = reinterpret_cast<FrontState*>(tp);
    uint8_t* codes_d = tp + off_codes;
    uint32_t* cnt_d = reinterpret_cast<uint32_t*>(tp + off_cnt);
    uint32_t* rowG = reinterpret_cast<uint32_t*>(tp + off_rows);
    uint32_t* rowN = rowG + m;
    uint32_t* rowP = rowN + m;
    uint32_t* rowPtrTmp = rowP + m;
    uint32_t* rowOffTmp = rowPtrTmp + m + 1;

    int rc = run_codes(W, N, m, n, codebook, K, bits, s, sd, codes_d, cnt_d, nullptr);
    if (rc != CER_OK) return rc;
    const unsigned row_blocks = (unsigned)((m + 3) / 4);
    const int64_t rows_per_block = 16;
    hist_kernel<<<(unsigned)((m + rows_per_block - 1) / rows_per_block), 256, 0, s>>>(cnt_d, m, rows_per_block, sd);
    rank_kernel<<<1, 256, 0, s>>>(sd);
    row_layout_kernel<<<row_blocks, 256, 0, s>>>(cnt_d, m, cser ? 1 : 0, sd, rowG, rowN, rowP);
    scan_rows_kernel<<<1, 1024, 0, s>>>(rowG, rowN, rowP, m, rowPtrTmp, rowOffTmp, sd);
    HIP_TRY(hipGetLastError());
    FrontState h;
    HIP_TRY(hipMemcpyAsync(&h, sd, sizeof h, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    rc = flags_to_error(h.flags);
    if (rc != CER_OK) return rc;
    if (K_out) *K_out = (int32_t)h.K;
    if (codebook_out) std::memcpy(codebook_out, h.codebook, (size_t)h.K * 4);

    // sizes are known: the handle's own allocation, filled in place by the emit kernel
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
    // the index arrays stay on the device until somebody asks for them on the host
    A->colI.len = A->nnz;
    A->colI.bits = min_index_bits(n > 0 ? (uint64_t)(n - 1) : 0);
    A->omegaPtr.len = A->G + 1;
    A->omegaPtr.bits = min_index_bits((uint64_t)A->nnz);
    A->rowPtr.len = m + 1;
    A->rowPtr.bits = min_index_bits((uint64_t)A->G);
    if (cser) {
        A->omegaI.len = A->G;
        A->omegaI.bits = min_index_bits(A->K > 0 ? (uint64_t)(A->K - 1) : 0);
    }
    A->arrays_on_host.store(false);
    const size_t colI_bytes = (size_t)A->nnz * (size_t)(A->colI.bits / 8);
    const size_t oi_bytes = cser ? (size_t)A->G * (size_t)(A->omegaI.bits / 8) : 0;
    const DeviceLayout l = DeviceLayout::make(colI_bytes, A->G, m, oi_bytes, A->K);
    void* base = nullptr;
    HIP_TRY(hipMalloc(&base, l.total));
    auto* b = static_cast<unsigned char*>(base);
    auto fail = [&](hipError_t e) {
        (void)hipStreamSynchronize(s);
        (void)hipFree(base);
        return record_hip_error((int)e);
    };
    // everything behind the indices is cleared (read-ahead padding, gaps); colI itself is written completely
    hipError_t e = hipMemsetAsync(b + colI_bytes, 0, l.total - colI_bytes, s);
    if (e == hipSuccess) e = hipMemcpyAsync(b + l.off_om, h.omega, (size_t)h.Kp * 4, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return fail(e);
    const int cs = cser ? 1 : 0;
    // with fewer than half of the elements indexed the emitter packs them in LDS before it scatters them
    const int sp = (double)A->nnz * 2.0 < (double)m * (double)n ? 1 : 0;
    switch (A->colI.bits) {
        case 8: launch_emit<uint8_t>(row_blocks, s, codes_d, cnt_d, rowPtrTmp, rowOffTmp, sd, m, n, cs, sp, b, l); break;
        case 16: launch_emit<uint16_t>(row_blocks, s, codes_d, cnt_d, rowPtrTmp, rowOffTmp, sd, m, n, cs, sp, b, l); break;
        default: launch_emit<uint32_t>(row_blocks, s, codes_d, cnt_d, rowPtrTmp, rowOffTmp, sd, m, n, cs, sp, b, l);
    }
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(s);  // `h.omega` lives on this frame; errors surface here
    if (e != hipSuccess) return fail(e);

    auto* hnd = new cer_matrix();
    hnd->host = std::move(A);
    bind_device(hnd, dev, base, l);
    e = (hipError_t)build_rank_table(hnd->view, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        cer_free(hnd);
        return record_hip_error((int)e);
    }
    // rows of unequal length: the batched product wants them ordered (and the longest in parts); the row starts
    // come back from the device only when the longest row says that the table will be built
    if (row_schedule_wanted((uint64_t)hnd->host->nnz, (uint64_t)m, (uint64_t)h.max_row_nnz)) {
        std::vector<uint32_t> info((size_t)(m + 1) * 2);
        e = hipMemcpy(info.data(), b + l.off_ri, info.size() * 4, hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            cer_free(hnd);
            return record_hip_error((int)e);
        }
        std::vector<uint64_t> start((size_t)m + 1);
        for (int64_t r = 0; r <= m; ++r) start[(size_t)r] = info[(size_t)r * 2 + 1];
        const int rc = build_row_schedule(hnd, start);
        if (rc != CER_OK) {
            cer_free(hnd);
            return rc;
        }
    }
    *out = hnd;
    return CER_OK;
}

}  // namespace cer
