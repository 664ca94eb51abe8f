// Dense fp32 product Y = W.X (Algorithm 1 of the paper) for gfx950: the baseline the CER / CSER
// speed-up is quoted against, plus a plain copy kernel used to calibrate memory-traffic counters.
//
//   batch = 1   one wave per two rows, 16-byte loads, DPP wave reduction: bound by the HBM read of W.
//   batch > 1   LDS-tiled GEMM on the fp32 matrix cores (v_mfma_f32_32x32x2f32), register-prefetched
//               double buffering, split along n when the output alone gives too few workgroups
//               (skinny batches), partial results summed by a second small kernel.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>

#include "cer_internal.hpp"

namespace cer {
namespace {

constexpr int kWave = 64;

__device__ __forceinline__ float wave_sum_dense(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
    return x;
}

template <int R>
__global__ __launch_bounds__(256) void dense_gemv_kernel(const float* __restrict__ W, const float* __restrict__ X,
                                                         float* __restrict__ Y, uint32_t m, uint32_t n, int vec_ok) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const uint32_t r0 = wave * R;
    if (r0 >= m) return;
    float acc[R];
#pragma unroll
    for (int k = 0; k < R; ++k) acc[k] = 0.f;
    const float* rows[R];
#pragma unroll
    for (int k = 0; k < R; ++k) rows[k] = W + (size_t)min(r0 + k, m - 1) * n;
    uint32_t c = 0;
    if (vec_ok) {
        const uint32_t n4 = n >> 2;
        const float4* X4 = reinterpret_cast<const float4*>(X);
        for (uint32_t i = lane; i < n4; i += kWave) {
            const float4 x = X4[i];
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const float4 w = reinterpret_cast<const float4*>(rows[k])[i];
                acc[k] = fmaf(w.x, x.x, acc[k]); acc[k] = fmaf(w.y, x.y, acc[k]);
                acc[k] = fmaf(w.z, x.z, acc[k]); acc[k] = fmaf(w.w, x.w, acc[k]);
            }
        }
        c = n4 << 2;
    }
    for (uint32_t i = c + lane; i < n; i += kWave) {
        const float x = X[i];
#pragma unroll
        for (int k = 0; k < R; ++k) acc[k] = fmaf(rows[k][i], x, acc[k]);
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const float y = wave_sum_dense(acc[k]);
        if (lane == 0 && r0 + k < m) Y[r0 + k] = y;
    }
}

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Block tile BM x BN, k-step 16 through LDS, 4 waves, each wave owns WM x WN outputs as (WM/32) x (WN/32)
// tiles of the 32x32x2 fp32 MFMA.  Out = Y, or one slab of the split-n workspace.
template <int BM, int BN, int WM, int WN, bool kVec>
__global__ __launch_bounds__(256) void dense_gemm_mfma_kernel(const float* __restrict__ W, const float* __restrict__ X,
                                                              float* __restrict__ Out, uint32_t m, uint32_t n,
                                                              uint32_t L, uint32_t kchunk, size_t split_stride) {
    constexpr int BK = 16;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * WAVES_N == 4, "four waves per workgroup");
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_UNITS = BM * BK / 4 / 256;  // float4 units per thread
    constexpr int B_UNITS = (BK * BN / 4 + 255) / 256;
    __shared__ float As[2][BK][BM + 4];
    __shared__ float Bs[2][BK][BN + 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const uint32_t row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    const uint32_t k_begin = blockIdx.z * kchunk, k_end = min(n, k_begin + kchunk);
    Out += (size_t)blockIdx.z * split_stride;

    float4 ra[A_UNITS], rb[B_UNITS];
    const bool full_mn = kVec && row0 + BM <= m && col0 + BN <= L;  // uniform over the workgroup
    auto fetch = [&](uint32_t k0) {
        if (full_mn && k0 + BK <= k_end) {
            // interior tile: no bounds to check
#pragma unroll
            for (int i = 0; i < A_UNITS; ++i) {
                const int u = tid + i * 256;
                ra[i] = *reinterpret_cast<const float4*>(W + (size_t)(row0 + u / 4) * n + k0 + (u % 4) * 4);
            }
#pragma unroll
            for (int i = 0; i < B_UNITS; ++i) {
                const int u = tid + i * 256;
                if (u < BK * BN / 4)
                    rb[i] = *reinterpret_cast<const float4*>(X + (size_t)(k0 + u / (BN / 4)) * L + col0 + (u % (BN / 4)) * 4);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) {
            const int u = tid + i * 256;
            const uint32_t r = row0 + u / 4, k = k0 + (u % 4) * 4;
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (r < m) {
                const float* p = W + (size_t)r * n + k;
                if (kVec && k + 3 < k_end) {
                    t = *reinterpret_cast<const float4*>(p);
                } else {
                    if (k < k_end) t.x = p[0];
                    if (k + 1 < k_end) t.y = p[1];
                    if (k + 2 < k_end) t.z = p[2];
                    if (k + 3 < k_end) t.w = p[3];
                }
            }
            ra[i] = t;
        }
#pragma unroll
        for (int i = 0; i < B_UNITS; ++i) {
            const int u = tid + i * 256;
            const uint32_t k = k0 + u / (BN / 4), c = col0 + (u % (BN / 4)) * 4;
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u < BK * BN / 4 && k < k_end) {
                const float* p = X + (size_t)k * L + c;
                if (kVec && c + 3 < L) {
                    t = *reinterpret_cast<const float4*>(p);
                } else {
                    if (c < L) t.x = p[0];
                    if (c + 1 < L) t.y = p[1];
                    if (c + 2 < L) t.z = p[2];
                    if (c + 3 < L) t.w = p[3];
                }
            }
            rb[i] = t;
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_UNITS; ++i) {
            const int u = tid + i * 256;
            const int r = u / 4, k = (u % 4) * 4;
            As[buf][k + 0][r] = ra[i].x; As[buf][k + 1][r] = ra[i].y;
            As[buf][k + 2][r] = ra[i].z; As[buf][k + 3][r] = ra[i].w;
        }
#pragma unroll
        for (int i = 0; i < B_UNITS; ++i) {
            const int u = tid + i * 256;
            if (u < BK * BN / 4) {
                const int k = u / (BN / 4), c = (u % (BN / 4)) * 4;
                *reinterpret_cast<float4*>(&Bs[buf][k][c]) = rb[i];
            }
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    int buf = 0;
    if (k_begin < k_end) {
        fetch(k_begin);
        stash(0);
    }
    __syncthreads();
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
        const bool more = k0 + BK < k_end;
        if (more) fetch(k0 + BK);
        // operands of the next pair of n-steps are read from LDS while the matrix cores work on the current pair; the
        // next tile goes to the other LDS buffer three quarters through, under the last products
        float a[2][TM], b[2][TN];
        auto frag = [&](int kk, int slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i) a[slot][i] = As[buf][kk + (lane >> 5)][wm * WM + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[slot][j] = Bs[buf][kk + (lane >> 5)][wn * WN + j * 32 + (lane & 31)];
        };
        frag(0, 0);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const int cur = (kk >> 1) & 1;
            if (kk + 2 < BK) frag(kk + 2, cur ^ 1);
            if (kk == (3 * BK) / 4 && more) stash(buf ^ 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
        buf ^= 1;
    }

    // accumulator element e of lane l: row = 8 (e / 4) + 4 (l / 32) + e % 4, column = l % 32
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const uint32_t c = col0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const uint32_t r = row0 + wm * WM + i * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e % 4);
                if (r < m && c < L) Out[(size_t)r * L + c] = acc[i][j][e];
            }
        }
}

__global__ __launch_bounds__(256) void split_sum_kernel(const float* __restrict__ part, float* __restrict__ Y,
                                                        size_t count, uint32_t splits) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float a = 0.f, b = 0.f;
    uint32_t s = 0;
    for (; s + 1 < splits; s += 2) {
        a += part[(size_t)s * count + i];
        b += part[(size_t)(s + 1) * count + i];
    }
    if (s < splits) a += part[(size_t)s * count + i];
    Y[i] = a + b;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Reads n16 16-byte pieces and keeps the loads alive by folding them into one word per wave.
// Launch shape of the batch-1 product kernel (256 workgroups of 1024 threads): what a kernel that
// does nothing but stream the same number of bytes costs.
__global__ __launch_bounds__(1024) void stream_read_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 1024;
    size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc ^= (uint32_t)__shfl_xor((int)acc, off, 64);
    if ((threadIdx.x & 63u) == 0) sink[blockIdx.x * 16u + (threadIdx.x >> 6)] = acc;
}

// Compute units of the current device (256 on MI355X).
int compute_units() {
    static int units[16];
    static std::once_flag once[16];
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 16) dev = 0;
    std::call_once(once[dev], [dev] {
        hipDeviceProp_t p;
        units[dev] = (hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0) ? p.multiProcessorCount : 256;
    });
    return units[dev];
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_gemm_cfg(const float* W, const float* X, float* Y, uint32_t m, uint32_t n, uint32_t L,
                           hipStream_t stream) {
    const bool vec = (n % 4 == 0) && (L % 4 == 0) && ((reinterpret_cast<uintptr_t>(W) & 15u) == 0) &&
                     ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);
    const uint32_t gx = (L + BN - 1) / BN, gy = (m + BM - 1) / BM;
    // Split along n so that the workgroups spread evenly over the compute units: the kernel lasts as long as the
    // busiest unit, rounds = ceil(workgroups / units) workgroups of ksteps / splits steps each.  A second workgroup
    // per unit hides the first one's waits; every split costs a partial result written and read again.
    uint32_t splits = 1;
    const uint32_t tiles = gx * gy, ksteps = (n + 15) / 16;
    if (tiles < 1024) {
        const uint32_t units = (uint32_t)std::max(compute_units(), 1);
        const uint32_t max_splits = std::min<uint32_t>(32u, std::max<uint32_t>(ksteps / 8, 1u));
        const double step_cycles = (WM / 32) * (WN / 32) * 8 * 64.0;  // matrix-core cycles per step and wave
        double best = 1e300;
        for (uint32_t sp = 1; sp <= max_splits; ++sp) {
            const uint32_t rounds = (tiles * sp + units - 1) / units;
            const uint32_t steps = (ksteps + sp - 1) / sp;
            double cost = (double)rounds * steps * step_cycles * (rounds == 1 ? 1.35 : 1.0);
            // the partial sums: one more launch, and about 6 bytes per cycle and unit written and read again
            if (sp > 1) cost += 7000.0 + (double)sp * BM * BN * 8.0 * ((double)tiles / units) / 6.0;
            if (cost < best) {
                best = cost;
                splits = sp;
            }
        }
    }
    const uint32_t kchunk = ((ksteps + splits - 1) / splits) * 16;
    splits = (n + kchunk - 1) / kchunk;
    if (splits < 1) splits = 1;
    float* part = nullptr;
    const size_t count = (size_t)m * L;
    hipError_t e = hipSuccess;
    if (splits > 1) {
        e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&part), count * splits * sizeof(float), stream);
        if (e != hipSuccess) return e;
    }
    float* out = splits > 1 ? part : Y;
    if (vec)
        hipLaunchKernelGGL((dense_gemm_mfma_kernel<BM, BN, WM, WN, true>), dim3(gx, gy, splits), dim3(256), 0, stream, W, X,
                           out, m, n, L, kchunk, count);
    else
        hipLaunchKernelGGL((dense_gemm_mfma_kernel<BM, BN, WM, WN, false>), dim3(gx, gy, splits), dim3(256), 0, stream, W,
                           X, out, m, n, L, kchunk, count);
    e = hipGetLastError();
    if (splits > 1) {
        if (e == hipSuccess) {
            hipLaunchKernelGGL(split_sum_kernel, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, stream, part, Y, count,
                               splits);
            e = hipGetLastError();
        }
        hipError_t f = (hipError_t)temp_free(part, stream);
        if (e == hipSuccess) e = f;
    }
    return e;
}

}  // namespace

int launch_dense(const float* W, const float* X, float* Y, int64_t m, int64_t n, int64_t L, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (m == 0) return (int)hipSuccess;
    if (m > 0x7FFFFFFFll || n > 0x7FFFFFFFll || L > 0x7FFFFFFFll || m * L > 0x7FFFFFFFFFll) return (int)hipErrorInvalidValue;
    if (L == 1) {
        constexpr int R = 2;
        const int vec_ok = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(W) & 15u) == 0) &&
                           ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);
        const uint32_t waves = (uint32_t)((m + R - 1) / R);
        hipLaunchKernelGGL(dense_gemv_kernel<R>, dim3((waves + 3) / 4), dim3(256), 0, stream, W, X, Y, (uint32_t)m,
                           (uint32_t)n, vec_ok);
        return (int)hipGetLastError();
    }
    if (L <= 32) return (int)launch_gemm_cfg<128, 32, 32, 32>(W, X, Y, (uint32_t)m, (uint32_t)n, (uint32_t)L, stream);
    // 128 x 64 tiles also for wide batches: measured 3 - 8 % ahead of 128 x 128 (more workgroups per compute unit)
    return (int)launch_gemm_cfg<128, 64, 32, 64>(W, X, Y, (uint32_t)m, (uint32_t)n, (uint32_t)L, stream);
}

int launch_stream_copy(void* dst, const void* src, int64_t bytes, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const size_t n16 = (size_t)bytes / 16;
    if (n16 == 0) return (int)hipSuccess;
    const uint32_t blocks = (uint32_t)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(stream_copy_kernel, dim3(blocks), dim3(256), 0, stream, static_cast<const uint4*>(src),
                       static_cast<uint4*>(dst), n16);
    return (int)hipGetLastError();
}

int launch_stream_read(const void* src, int64_t bytes, void* sink, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    hipLaunchKernelGGL(stream_read_kernel, dim3(256), dim3(1024), 0, stream, static_cast<const uint4*>(src),
                       (size_t)bytes / 16, static_cast<uint32_t*>(sink));
    return (int)hipGetLastError();
}

}  // namespace cer
