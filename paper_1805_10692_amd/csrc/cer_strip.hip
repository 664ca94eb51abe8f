// Batch > 1 with strips of X resident in LDS: the reuse of input elements that Section V-C of the paper names as the
// missing optimisation, in its column-blocked form.
//
// The kernels that gather rows of X from L2 are bound by the compute unit's vector-memory pipeline (about 26 clocks
// per wave instruction of 1 KB, i.e. 40 bytes per clock); LDS delivers 128 bytes per clock.  Here the input is cut
// into strips of 1024 consecutive rows; a workgroup copies one strip of one tile of 32 batch columns into LDS
// (128 KB, rows of 128 bytes) and serves from it every indexed element of its rows of W whose column falls into the
// strip.  The format orders a row's indices by value, then column, so a strip's share of a row is scattered over
// the row's groups: the handle carries a DERIVED strip-major index (built once by cer_prepare_strips from the format
// arrays; 2 bytes per indexed element, the same as colI, plus one 32-bit pointer per strip and row), whose entries
// hold the column inside the strip (10 bits) and the rank of the element's value (6 bits: codebooks of at most 64
// values).  Every element is multiplied by its own value (Omega[rank] - Omega[0] from a table in LDS), so the
// fragmentation of the groups does not matter.  The eight 8-lane parts of a wave take eight different rows of W, so
// no cross-lane reduction is needed; one gather instruction reads eight 128-byte rows of the strip without bank
// conflicts.  Each (strip, row) leaves a partial sum; a second kernel adds the strips' partial sums in strip order
// (deterministic) and the constant term of a non-zero most frequent value (Appendix A-A1).
#include "cer_device.hpp"

namespace cer {
namespace {

constexpr uint32_t kStripTile = 32;  // batch columns per tile: one 128-byte row of the strip per index

typedef float F4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(1024) void cer_strip_kernel(const uint16_t* __restrict__ sidx, const uint32_t* __restrict__ sptr,
                                                         const float* __restrict__ X, float* __restrict__ part,
                                                         const float* __restrict__ omega, uint32_t m, uint32_t n, uint32_t L,
                                                         uint32_t K, float omega0, uint32_t ntiles, uint32_t nsplit,
                                                         uint32_t rows_per_split) {
    extern __shared__ __align__(16) unsigned char strip_smem[];
    __shared__ float s_w[64];
    F4* xs4 = reinterpret_cast<F4*>(strip_smem);  // [rows of the strip][8 x 16 bytes]
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = uniform(threadIdx.x >> 6);
    const uint32_t split = blockIdx.x % nsplit, tile = (blockIdx.x / nsplit) % ntiles, s = blockIdx.x / (nsplit * ntiles);
    const uint32_t c0 = s * kStripRows, rows_here = min(kStripRows, n - c0);

    // the strip of this tile of batch columns: 8 threads copy one 128-byte row
    const F4* X4 = reinterpret_cast<const F4*>(X);
    const uint32_t row_f4 = L >> 2;  // 16-byte pieces per row of X
    for (uint32_t i = threadIdx.x; i < rows_here * 8u; i += blockDim.x)
        xs4[i] = X4[(size_t)(c0 + (i >> 3)) * row_f4 + tile * 8u + (i & 7u)];
    if (threadIdx.x < 64u) s_w[threadIdx.x] = threadIdx.x < K ? omega[threadIdx.x] - omega0 : 0.f;
    __syncthreads();

    const uint32_t r_begin = split * rows_per_split, r_end = min(m, r_begin + rows_per_split);
    const uint32_t sub = lane >> 3, ch = lane & 7u;
    const uint32_t* sp = sptr + (size_t)s * (m + 1);
    const int lane0 = (int)(lane & ~7u);  // the first lane of this lane's 8-lane part
    for (uint32_t r0 = r_begin + wave * 8u; r0 < r_end; r0 += (blockDim.x >> 6) * 8u) {  // wave-uniform
        const uint32_t r = r0 + sub;
        const bool row_ok = r < r_end;
        const uint32_t e0 = row_ok ? sp[r] : 0u, e1 = row_ok ? sp[r + 1] : 0u;
        const uint32_t nent = e1 - e0;
        F4 acc = F4{0.f, 0.f, 0.f, 0.f};
        for (uint32_t it = 0; __ballot(it < nent) != 0ull; it += 8u) {
            // the part's next eight entries, one per lane; then each of them is handed to all eight lanes in turn
            const uint32_t left = it < nent ? nent - it : 0u;
            const uint32_t ent = ch < left ? (uint32_t)sidx[e0 + it + ch] : 0u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t e = (uint32_t)__shfl((int)ent, lane0 + i, kWave);
                const float w = (uint32_t)i < left ? s_w[e >> 10] : 0.f;
                const F4 x = xs4[(e & 1023u) * 8u + ch];
                acc.x = fmaf(w, x.x, acc.x); acc.y = fmaf(w, x.y, acc.y);
                acc.z = fmaf(w, x.z, acc.z); acc.w = fmaf(w, x.w, acc.w);
            }
        }
        if (row_ok) reinterpret_cast<F4*>(part)[((size_t)s * m + r) * row_f4 + tile * 8u + ch] = acc;
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

}  // namespace

bool strip_applicable(const DeviceView& d, const float* X, const float* Y, uint32_t L) {
    return d.strip_idx != nullptr && d.n_strips > 0 && L >= kStripTile && L % kStripTile == 0 && d.m > 0 &&
           (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && (reinterpret_cast<uintptr_t>(Y) & 15u) == 0 &&
           d.lds_per_block >= (size_t)kStripRows * kStripTile * 4 + 1024;
}

hipError_t launch_strip(const DeviceView& d, const float* X, float* Y, const float* T, uint32_t L, hipStream_t stream) {
    const uint32_t m = (uint32_t)d.m, n = (uint32_t)d.n, ntiles = L / kStripTile;
    // enough workgroups for every compute unit, each with at least 64 rows: the rows are split over `nsplit` workgroups
    const uint64_t base = (uint64_t)d.n_strips * ntiles;
    uint32_t nsplit = (uint32_t)std::max<uint64_t>(1, (2ull * (uint64_t)d.cus + base - 1) / base);
    nsplit = std::min<uint32_t>(nsplit, std::max<uint32_t>(1u, m / 64u));
    const uint32_t rows_per_split = (((m + nsplit - 1) / nsplit) + 7u) & ~7u;
    nsplit = (m + rows_per_split - 1) / rows_per_split;
    const uint64_t blocks = base * nsplit;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    float* part = nullptr;
    const size_t part_bytes = (size_t)d.n_strips * m * L * sizeof(float);
    hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&part), part_bytes, stream);
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)kStripRows * kStripTile * sizeof(float);
    static LdsGrant<1> grant;
    e = grant.ensure(0, reinterpret_cast<const void*>(cer_strip_kernel), d.lds_per_block - 512);  // less the static words
    if (e == hipSuccess) {
        hipLaunchKernelGGL(cer_strip_kernel, dim3((uint32_t)blocks), dim3(1024), lds, stream,
                           static_cast<const uint16_t*>(d.strip_idx), d.strip_ptr, X, part, d.omega, m, n, L, (uint32_t)d.K,
                           d.omega0, ntiles, nsplit, rows_per_split);
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
