// CSR comparator (Section III-A "Sparse format" and Algorithm 2 of the paper) in the same harness as
// the CER / CSER path: host encoder / decoder, device upload, and the product kernels.
//
// The kernels mirror the CER ones so that the comparison isolates the format: one wave per row,
// consecutive positions per wave instruction, X staged in LDS for batch 1, lanes across the batch
// columns for batch > 1 -- but every stored element brings its own fp32 value (6 bytes per element
// instead of 2) and costs one multiply-add, where CER / CSER multiply once per group.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/cer.h"
#include "cer_internal.hpp"

namespace {

constexpr int kWave = 64;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

// batch = 1.  Same treatment as the CER batch-1 kernel, so that the comparison isolates the format: what bounds a
// launch of this size is the number of vector-memory instructions a compute unit issues, so values and indices are
// read with wide loads (a lane holds 4 consecutive elements of a window of 256: one 16-byte load of values, one load
// of 4 indices), four windows in flight, a batch starting at a multiple of 4 elements (aligned loads); X is staged
// into LDS with 16-byte loads.  colI and the values are followed by readable padding, so all loads of a batch are
// unconditional; elements in front of the row or past its end are given the value 0.
constexpr int kCsrWindows = 4;  // windows of 256 elements in flight per wave

template <typename IdxT>
__device__ __forceinline__ void csr_load_indices(const IdxT* p, uint32_t (&idx)[4]) {  // p is 4-element aligned
    if (sizeof(IdxT) == 4) {
        const uint4 q = *reinterpret_cast<const uint4*>(p);
        idx[0] = q.x; idx[1] = q.y; idx[2] = q.z; idx[3] = q.w;
    } else if (sizeof(IdxT) == 2) {
        const uint2 q = *reinterpret_cast<const uint2*>(p);
        idx[0] = q.x & 0xFFFFu; idx[1] = q.x >> 16; idx[2] = q.y & 0xFFFFu; idx[3] = q.y >> 16;
    } else {
        const uint32_t q = *reinterpret_cast<const uint32_t*>(p);
        idx[0] = q & 0xFFu; idx[1] = (q >> 8) & 0xFFu; idx[2] = (q >> 16) & 0xFFu; idx[3] = q >> 24;
    }
}

template <typename IdxT, bool kXinLds>
__global__ __launch_bounds__(1024) void csr_gemv_kernel(const float* __restrict__ val, const IdxT* __restrict__ colI,
                                                        const uint32_t* __restrict__ rowPtr, const float* __restrict__ X,
                                                        float* __restrict__ Y, uint32_t m, uint32_t n,
                                                        uint32_t rows_per_block) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* xs = reinterpret_cast<float*>(smem);
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t nwaves = blockDim.x >> 6;
    if (kXinLds) {
        if ((reinterpret_cast<uintptr_t>(X) & 15u) == 0) {
            const uint32_t n4 = n >> 2;
            const float4* X4 = reinterpret_cast<const float4*>(X);
            float4* xs4 = reinterpret_cast<float4*>(xs);
            for (uint32_t i = threadIdx.x; i < n4; i += blockDim.x) xs4[i] = X4[i];
            for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += blockDim.x) xs[i] = X[i];
        } else {
            for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) xs[i] = X[i];
        }
        __syncthreads();
    }
    const float* xsrc = kXinLds ? xs : X;
    const uint32_t row_begin = blockIdx.x * rows_per_block;
    const uint32_t row_end = min(m, row_begin + rows_per_block);
    for (uint32_t r = row_begin + wave; r < row_end; r += nwaves) {
        const uint32_t rs = rowPtr[r], re = rowPtr[r + 1];
        float acc0 = 0.f, acc1 = 0.f;
        for (uint32_t b0 = rs & ~3u; b0 < re; b0 += kCsrWindows * 4 * kWave) {
            float4 w[kCsrWindows];
            uint32_t idx[kCsrWindows][4];
#pragma unroll
            for (int W = 0; W < kCsrWindows; ++W) {
                const uint32_t pos = b0 + (uint32_t)W * 4u * kWave + 4u * lane;
                w[W] = *reinterpret_cast<const float4*>(val + pos);
                csr_load_indices<IdxT>(colI + pos, idx[W]);
            }
#pragma unroll
            for (int W = 0; W < kCsrWindows; ++W) {
                if (W > 0 && b0 + (uint32_t)W * 4u * kWave >= re) break;  // wave-uniform
                const uint32_t pos = b0 + (uint32_t)W * 4u * kWave + 4u * lane;
                const float x0 = xsrc[idx[W][0]], x1 = xsrc[idx[W][1]], x2 = xsrc[idx[W][2]], x3 = xsrc[idx[W][3]];
                acc0 = fmaf((pos >= rs && pos < re) ? w[W].x : 0.f, x0, acc0);
                acc1 = fmaf((pos + 1u >= rs && pos + 1u < re) ? w[W].y : 0.f, x1, acc1);
                acc0 = fmaf((pos + 2u >= rs && pos + 2u < re) ? w[W].z : 0.f, x2, acc0);
                acc1 = fmaf((pos + 3u >= rs && pos + 3u < re) ? w[W].w : 0.f, x3, acc1);
            }
        }
        const float y = wave_sum(acc0 + acc1);
        if (lane == 0) Y[r] = y;
    }
}

// batch > 1: P lanes x 4 floats (or 1 float when the batch is not a multiple of 4) cover a tile of
// batch columns, the wave's 64/P sub-groups take consecutive elements.
template <int P>
struct CsrIdx {  // one register = 64 consecutive positions; a batch of U windows covers PB positions = KQ registers
    static constexpr int S = kWave / P, U = 8, PB = U * S;
    static constexpr int KQ = PB >= kWave ? PB / kWave : 1;
    static constexpr int D = KQ == 1 ? 8 : (KQ <= 4 ? 4 : 2);  // batches of (index, value) registers in flight
};

// Same streaming structure as the CER batched kernel, so that the comparison isolates the format: indices AND
// values are fetched with one coalesced load per 64 positions each and handed to the lanes by cross-lane reads,
// D batches ahead; two batches of gathers are in flight; every gathered row is multiplied by its element's value.
template <typename IdxT, int V, int P>
__global__ __launch_bounds__(256) void csr_gemm_kernel(const float* __restrict__ val, const IdxT* __restrict__ colI,
                                                       const uint32_t* __restrict__ rowPtr, const float* __restrict__ X,
                                                       float* __restrict__ Y, uint32_t m, uint32_t L, uint32_t ntiles,
                                                       uint32_t rowblocks, uint32_t items_per_xcd) {
    using G = CsrIdx<P>;
    constexpr int S = G::S, U = G::U, KQ = G::KQ, D = G::D, TW = V * P;
    constexpr uint32_t PB = G::PB;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t xcd = blockIdx.x & 7u, q = blockIdx.x >> 3;
    const uint32_t item = xcd * items_per_xcd + q;
    if (q >= items_per_xcd || item >= ntiles * rowblocks) return;
    const uint32_t tile = item / rowblocks;
    const uint32_t r = (item - tile * rowblocks) * 4u + wave;
    if (r >= m) return;
    const uint32_t sub = lane / P;
    const uint32_t col0 = tile * TW + (lane % P) * V;
    const bool active = col0 < L;
    const float* xg = X + (active ? col0 : 0u);
    const uint32_t rs = rowPtr[r], re = rowPtr[r + 1];
    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.f;

    uint32_t iq[D][KQ];
    float vq[D][KQ];
    float xa[U][V], xb[U][V], wa[U], wb[U];
#define CSR_LOADQ(d, b)                                             \
    _Pragma("unroll") for (int qq = 0; qq < KQ; ++qq) {             \
        iq[d][qq] = (uint32_t)colI[(b) + qq * kWave + lane];        \
        vq[d][qq] = val[(b) + qq * kWave + lane];                   \
    }
#define CSR_GATHER(xv, wv, d)                                                                          \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                                    \
        const int src_ = (int)((u * S) % kWave + sub);                                                 \
        const uint32_t idx_ = S == kWave ? iq[d][(u * S) / kWave] : (uint32_t)__shfl((int)iq[d][(u * S) / kWave], src_, kWave); \
        wv[u] = S == kWave ? vq[d][(u * S) / kWave] : __shfl(vq[d][(u * S) / kWave], src_, kWave);     \
        const float* p_ = xg + (size_t)idx_ * L;                                                       \
        if (V == 4) {                                                                                  \
            const float4 t_ = *reinterpret_cast<const float4*>(p_);                                    \
            xv[u][0] = t_.x; xv[u][1 % V] = t_.y; xv[u][2 % V] = t_.z; xv[u][3 % V] = t_.w;            \
        } else {                                                                                       \
            xv[u][0] = p_[0];                                                                          \
        }                                                                                              \
    }
#define CSR_CONSUME(xv, wv, b)                                                         \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                    \
        const float w_ = ((b) + u * S + sub < re) ? wv[u] : 0.f; /* past the row */    \
        _Pragma("unroll") for (int k = 0; k < V; ++k) acc[k] = fmaf(w_, xv[u][k], acc[k]); \
    }
#define CSR_STEP(xcur, wcur, xnext, wnext, dn, dl, k) \
    CSR_GATHER(xnext, wnext, dn)                      \
    CSR_LOADQ(dl, base + ((k) + D) * PB)              \
    CSR_CONSUME(xcur, wcur, base + (k) * PB)
#pragma unroll
    for (int d = 0; d < D; ++d) { CSR_LOADQ(d, rs + d * PB) }
    CSR_GATHER(xa, wa, 0)
    for (uint32_t base = rs; base < re; base += D * PB) {
        CSR_STEP(xa, wa, xb, wb, 1 % D, 0, 0)
        if (D > 2 && base + PB >= re) break;
        CSR_STEP(xb, wb, xa, wa, 2 % D, 1 % D, 1)
        if (D > 2) {
            if (base + 2 * PB >= re) break;
            CSR_STEP(xa, wa, xb, wb, 3 % D, 2 % D, 2)
            if (base + 3 * PB >= re) break;
            CSR_STEP(xb, wb, xa, wa, 4 % D, 3 % D, 3)
        }
        if (D > 4) {
            if (base + 4 * PB >= re) break;
            CSR_STEP(xa, wa, xb, wb, 5 % D, 4 % D, 4)
            if (base + 5 * PB >= re) break;
            CSR_STEP(xb, wb, xa, wa, 6 % D, 5 % D, 5)
            if (base + 6 * PB >= re) break;
            CSR_STEP(xa, wa, xb, wb, 7 % D, 6 % D, 6)
            if (base + 7 * PB >= re) break;
            CSR_STEP(xb, wb, xa, wa, 0, 7 % D, 7)
        }
    }
#undef CSR_LOADQ
#undef CSR_GATHER
#undef CSR_CONSUME
#undef CSR_STEP
#pragma unroll
    for (int off = P; off < kWave; off <<= 1)
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] += __shfl_xor(acc[k], off, kWave);
    if (sub == 0 && active) {
#pragma unroll
        for (int k = 0; k < V; ++k) Y[(size_t)r * L + col0 + k] = acc[k];
    }
}

struct DevInfo {
    int cus = 256;
    size_t lds = 64 * 1024;
};

DevInfo dev_info() {
    DevInfo d;
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) {
        d.cus = p.multiProcessorCount > 0 ? p.multiProcessorCount : 256;
        d.lds = std::max<size_t>(p.sharedMemPerBlock, p.maxSharedMemoryPerMultiProcessor);
    }
    return d;
}

template <typename IdxT>
hipError_t launch_gemv(const csr_matrix& h, const float* X, float* Y, hipStream_t stream) {
    static const DevInfo di = dev_info();
    const uint32_t m = (uint32_t)h.host->m, n = (uint32_t)h.host->n;
    const size_t x_bytes = (size_t)n * 4;
    const bool x_in_lds = x_bytes <= di.lds;
    // as for the CER batch-1 kernel: an X of tens of kilobytes is staged once per compute unit
    int waves = 4;
    if (x_in_lds && x_bytes > 24 * 1024) {
        const uint32_t per_unit = (m + (uint32_t)di.cus - 1) / (uint32_t)di.cus;
        uint32_t w2 = 4;
        while (w2 < per_unit && w2 < 16) w2 <<= 1;
        waves = (int)w2;
    }
    const size_t lds = x_in_lds ? x_bytes : 0;
    size_t per_cu = std::min<size_t>(lds ? di.lds / lds : 8, (size_t)(32 / waves));
    per_cu = std::max<size_t>(1, std::min<size_t>(per_cu, 8));
    const uint64_t slots = (uint64_t)di.cus * per_cu;
    const uint32_t iters = std::max<uint32_t>(1u, (uint32_t)((m + slots * waves - 1) / (slots * waves)));
    const uint32_t rows_per_block = iters * waves;
    const uint32_t blocks = (m + rows_per_block - 1) / rows_per_block;
    auto kern = x_in_lds ? csr_gemv_kernel<IdxT, true> : csr_gemv_kernel<IdxT, false>;
    if (lds > 48 * 1024) {
        static std::once_flag once;
        static hipError_t err = hipSuccess;
        std::call_once(once, [&] {
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(csr_gemv_kernel<IdxT, true>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)di.lds);
        });
        if (err != hipSuccess) return err;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, stream, h.d_val, static_cast<const IdxT*>(h.d_colI),
                       h.d_rowPtr, X, Y, m, n, rows_per_block);
    return hipGetLastError();
}

template <typename IdxT, int V, int P>
hipError_t launch_gemm_vp(const csr_matrix& h, const float* X, float* Y, uint32_t L, hipStream_t stream) {
    const uint32_t m = (uint32_t)h.host->m;
    const uint32_t ntiles = (L + V * P - 1) / (V * P), rowblocks = (m + 3) / 4;
    const uint64_t nitems = (uint64_t)ntiles * rowblocks;
    if (nitems > 0x7FFFFFFFull / 8) return hipErrorInvalidValue;
    const uint32_t ipx = (uint32_t)((nitems + 7) / 8);
    hipLaunchKernelGGL((csr_gemm_kernel<IdxT, V, P>), dim3(ipx * 8), dim3(256), 0, stream, h.d_val,
                       static_cast<const IdxT*>(h.d_colI), h.d_rowPtr, X, Y, m, L, ntiles, rowblocks, ipx);
    return hipGetLastError();
}

inline uint32_t pow2_ceil(uint32_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

template <typename IdxT>
hipError_t launch_any(const csr_matrix& h, const float* X, float* Y, uint32_t L, hipStream_t stream) {
    if (L == 1) return launch_gemv<IdxT>(h, X, Y, stream);
    const bool vec4 = (L % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);
    if (vec4) {
        switch (std::max<uint32_t>(4u, std::min<uint32_t>(pow2_ceil(L), 32u))) {
            case 4: return launch_gemm_vp<IdxT, 4, 1>(h, X, Y, L, stream);
            case 8: return launch_gemm_vp<IdxT, 4, 2>(h, X, Y, L, stream);
            case 16: return launch_gemm_vp<IdxT, 4, 4>(h, X, Y, L, stream);
            default: return launch_gemm_vp<IdxT, 4, 8>(h, X, Y, L, stream);
        }
    }
    switch (std::min<uint32_t>(pow2_ceil(L), 64u)) {
        case 1: case 2: return launch_gemm_vp<IdxT, 1, 2>(h, X, Y, L, stream);
        case 4: return launch_gemm_vp<IdxT, 1, 4>(h, X, Y, L, stream);
        case 8: return launch_gemm_vp<IdxT, 1, 8>(h, X, Y, L, stream);
        case 16: return launch_gemm_vp<IdxT, 1, 16>(h, X, Y, L, stream);
        case 32: return launch_gemm_vp<IdxT, 1, 32>(h, X, Y, L, stream);
        default: return launch_gemm_vp<IdxT, 1, 64>(h, X, Y, L, stream);
    }
}

// One allocation: [values | 8 KiB pad][colI | 8 KiB pad][rowPtr u32].
int upload(csr_matrix* h) {
    const csr_host& A = *h->host;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return CER_OK;  // host-only handle
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return cer::record_hip_error((int)e);
    const size_t val_bytes = (size_t)A.nnz * 4, idx_bytes = A.colI.bytes.size();
    const size_t off_idx = align_up(val_bytes + 8192, 256);
    const size_t off_rp = align_up(off_idx + idx_bytes + 8192, 256);
    const size_t total = align_up(off_rp + (size_t)(A.m + 1) * 4, 256);
    void* base = nullptr;
    e = hipMalloc(&base, total);
    if (e != hipSuccess) return cer::record_hip_error((int)e);
    auto* b = static_cast<unsigned char*>(base);
    e = hipMemset(base, 0, total);
    if (e == hipSuccess && val_bytes) e = hipMemcpy(b, A.val.data(), val_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess && idx_bytes) e = hipMemcpy(b + off_idx, A.colI.bytes.data(), idx_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        std::vector<uint32_t> rp((size_t)A.m + 1);
        for (int64_t r = 0; r <= A.m; ++r) rp[(size_t)r] = (uint32_t)A.rowPtr.at(r);
        e = hipMemcpy(b + off_rp, rp.data(), rp.size() * 4, hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        (void)hipFree(base);
        return cer::record_hip_error((int)e);
    }
    h->device = dev;
    h->d_base = base;
    h->d_val = reinterpret_cast<const float*>(b);
    h->d_colI = b + off_idx;
    h->d_rowPtr = reinterpret_cast<const uint32_t*>(b + off_rp);
    h->stream_bytes = (int64_t)(val_bytes + idx_bytes + (size_t)(A.m + 1) * 4);
    return CER_OK;
}

void narrow_into(const std::vector<uint32_t>& src, int bits, cer::HostArray* dst) {
    dst->len = (int64_t)src.size();
    dst->bits = bits;
    dst->bytes.resize(src.size() * (size_t)(bits / 8));
    for (size_t i = 0; i < src.size(); ++i) {
        if (bits == 8) dst->bytes[i] = (uint8_t)src[i];
        else if (bits == 16) reinterpret_cast<uint16_t*>(dst->bytes.data())[i] = (uint16_t)src[i];
        else reinterpret_cast<uint32_t*>(dst->bytes.data())[i] = src[i];
    }
}

}  // namespace

extern "C" {

int csr_encode(const float* W, int64_t m, int64_t n, csr_handle_t** out) {
    if (!out) return CER_E_INVALID;
    *out = nullptr;
    if (m < 0 || n < 0 || (m > 0 && n > 0 && !W)) return CER_E_INVALID;
    if (m > 0x7FFFFFFFll || n > 0xFFFFFFFFll) return CER_E_TOO_LARGE;
    try {
        auto A = std::make_shared<csr_host>();
        A->m = m;
        A->n = n;
        std::vector<uint32_t> colI, rowPtr((size_t)m + 1, 0);
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                const float v = W[r * n + c];
                if (v != 0.0f) {
                    A->val.push_back(v);
                    colI.push_back((uint32_t)c);
                }
            }
            if (A->val.size() > 0xFFFFFFFFull - 65536) return CER_E_TOO_LARGE;
            rowPtr[(size_t)r + 1] = (uint32_t)A->val.size();
        }
        A->nnz = (int64_t)A->val.size();
        narrow_into(colI, cer::min_index_bits(n > 0 ? (uint64_t)(n - 1) : 0), &A->colI);
        narrow_into(rowPtr, cer::min_index_bits((uint64_t)A->nnz), &A->rowPtr);
        auto* h = new csr_matrix();
        h->host = std::move(A);
        const int rc = upload(h);
        if (rc != CER_OK) {
            delete h;
            return rc;
        }
        *out = h;
        return CER_OK;
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    }
}

int csr_matmul(const csr_handle_t* h, const float* X, float* Y, int64_t batch, void* stream_v) {
    if (!h || !X || !Y || batch < 1 || batch > 0x7FFFFFFFll) return CER_E_INVALID;
    if (h->device < 0 || !h->d_base) return cer::record_hip_error((int)hipErrorNoDevice);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return cer::record_hip_error((int)e);
    if (dev != h->device) return cer::record_hip_error((int)hipErrorInvalidDevice);
    if (h->host->m == 0) return CER_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    switch (h->host->colI.bits) {
        case 8: e = launch_any<uint8_t>(*h, X, Y, (uint32_t)batch, stream); break;
        case 16: e = launch_any<uint16_t>(*h, X, Y, (uint32_t)batch, stream); break;
        default: e = launch_any<uint32_t>(*h, X, Y, (uint32_t)batch, stream); break;
    }
    return e == hipSuccess ? CER_OK : cer::record_hip_error((int)e);
}

int csr_decode(const csr_handle_t* h, float* W) {
    if (!h) return CER_E_INVALID;
    const csr_host& A = *h->host;
    if (!W && A.m * A.n > 0) return CER_E_INVALID;
    std::fill(W, W + A.m * A.n, 0.0f);
    for (int64_t r = 0; r < A.m; ++r)
        for (int64_t i = (int64_t)A.rowPtr.at(r); i < (int64_t)A.rowPtr.at(r + 1); ++i)
            W[r * A.n + (int64_t)A.colI.at(i)] = A.val[(size_t)i];
    return CER_OK;
}

int csr_get_array(const csr_handle_t* h, int which, const void** host_ptr, int64_t* len, int32_t* elem_bits) {
    if (!h || !host_ptr || !len || !elem_bits) return CER_E_INVALID;
    const csr_host& A = *h->host;
    switch (which) {
        case 0: *host_ptr = A.val.data(); *len = A.nnz; *elem_bits = 32; return CER_OK;
        case 1: *host_ptr = A.colI.bytes.data(); *len = A.colI.len; *elem_bits = A.colI.bits; return CER_OK;
        case 2: *host_ptr = A.rowPtr.bytes.data(); *len = A.rowPtr.len; *elem_bits = A.rowPtr.bits; return CER_OK;
        default: return CER_E_INVALID;
    }
}

int64_t csr_storage_bits(const csr_handle_t* h) {
    if (!h) return CER_E_INVALID;
    const csr_host& A = *h->host;
    return A.nnz * 32 + A.colI.len * A.colI.bits + A.rowPtr.len * A.rowPtr.bits;
}

int64_t csr_device_bytes(const csr_handle_t* h) { return (h && h->device >= 0) ? h->stream_bytes : 0; }

int csr_clone_device(const csr_handle_t* h, csr_handle_t** out) {
    if (!h || !out) return CER_E_INVALID;
    *out = nullptr;
    try {
        auto* c = new csr_matrix();
        c->host = h->host;
        const int rc = upload(c);
        if (rc != CER_OK) {
            delete c;
            return rc;
        }
        *out = c;
        return CER_OK;
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    }
}

void csr_free(csr_handle_t* h) {
    if (!h) return;
    if (h->d_base) (void)hipFree(h->d_base);
    delete h;
}

}  // extern "C"
