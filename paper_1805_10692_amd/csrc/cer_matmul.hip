// cer_matmul / cser_matmul: choice of the product kernel for a handle and a batch width, the column sums of X for
// a non-zero most frequent value (Appendix A-A1), and the decode + dense route.
#include "cer_device.hpp"

// Workspace of the entry point that allocates nothing: one array per GPU, part of the loaded code object, so it
// exists from the moment the library is loaded on a device until the process ends.  Host code never uses the
// array's name as an address: the address on the current device comes from hipGetSymbolAddress, once per device.
// (No `used` attribute: it keeps the symbol local to the code object, where the runtime's look-up by name cannot find it.)
constexpr size_t kStaticWorkspaceFloats = 512 * 1024;  // 2 MiB
static __device__ __align__(256) float scratch[kStaticWorkspaceFloats];

namespace cer {
namespace {

// ------------------------------------------------------------------------------------------------
// Column sums of X (Appendix A-A1): T[l] = sum_i X[i,l], in two stages of short partial sums.
// ------------------------------------------------------------------------------------------------

// block (bx, by): columns [bx*CB, +CB), rows [by*slab, +slab).  CB divides 256.
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ X, uint32_t n, uint32_t L,
                                                             uint32_t CB, uint32_t slab, float* __restrict__ part) {
    __shared__ float red[256];
    const uint32_t cl = threadIdx.x % CB, rl = threadIdx.x / CB, RPB = 256u / CB;
    const uint32_t col = blockIdx.x * CB + cl;
    const uint32_t i0 = blockIdx.y * slab, i1 = min(n, i0 + slab);
    float a0 = 0.f, a1 = 0.f;
    if (col < L) {
        uint32_t i = i0 + rl;
        for (; i + RPB < i1; i += 2 * RPB) {
            a0 += X[(size_t)i * L + col];
            a1 += X[(size_t)(i + RPB) * L + col];
        }
        if (i < i1) a0 += X[(size_t)i * L + col];
    }
    red[threadIdx.x] = a0 + a1;
    __syncthreads();
    for (uint32_t s = RPB >> 1; s > 0; s >>= 1) {
        if (rl < s) red[threadIdx.x] += red[threadIdx.x + s * CB];
        __syncthreads();
    }
    if (rl == 0 && col < L) part[(size_t)blockIdx.y * L + col] = red[cl];
}

// The same for wide batches (L a multiple of 4, X 16-byte aligned): a thread owns four columns and reads them with
// 16-byte loads, four rows in flight.  block (bx, by): columns [bx*1024, +1024), rows [by*slab, +slab).
__global__ __launch_bounds__(256) void colsum_partial4_kernel(const float* __restrict__ X, uint32_t n, uint32_t L,
                                                              uint32_t slab, float* __restrict__ part) {
    typedef float F4 __attribute__((ext_vector_type(4)));
    const uint32_t col = (blockIdx.x * 256u + threadIdx.x) * 4u;
    if (col >= L) return;
    const uint32_t i0 = blockIdx.y * slab, i1 = min(n, i0 + slab);
    const F4* p = reinterpret_cast<const F4*>(X + col);
    const size_t pitch = L >> 2;
    F4 a0 = F4{0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
    uint32_t i = i0;
    for (; i + 4 <= i1; i += 4) {
        const F4 x0 = p[(size_t)i * pitch], x1 = p[(size_t)(i + 1) * pitch], x2 = p[(size_t)(i + 2) * pitch],
                 x3 = p[(size_t)(i + 3) * pitch];
        a0 += x0; a1 += x1; a2 += x2; a3 += x3;
    }
    for (; i < i1; ++i) a0 += p[(size_t)i * pitch];
    *reinterpret_cast<F4*>(part + (size_t)blockIdx.y * L + col) = (a0 + a1) + (a2 + a3);
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const float* __restrict__ part, uint32_t nslabs, uint32_t L,
                                                           float* __restrict__ T) {
    const uint32_t col = blockIdx.x * 256u + threadIdx.x;
    if (col >= L) return;
    const float* p = part + col;
    float a = 0.f;
    uint32_t s = 0;
    for (; s + 8 <= nslabs; s += 8) {  // eight slabs requested at a time, added in slab order
        float b[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) b[k] = p[(size_t)(s + k) * L];
#pragma unroll
        for (int k = 0; k < 8; ++k) a += b[k];
    }
    for (; s < nslabs; ++s) a += p[(size_t)s * L];
    T[col] = a;
}

hipError_t launch_colsum(const float* X, uint32_t n, uint32_t L, float* part, uint32_t nslabs, uint32_t slab,
                         uint32_t CB, float* T, hipStream_t stream) {
    const uint32_t coltiles = (L + CB - 1) / CB;
    if (L >= 1024u && L % 4u == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && (reinterpret_cast<uintptr_t>(part) & 15u) == 0)
        hipLaunchKernelGGL(colsum_partial4_kernel, dim3((L + 1023u) / 1024u, nslabs), dim3(256), 0, stream, X, n, L, slab, part);
    else
        hipLaunchKernelGGL(colsum_partial_kernel, dim3(coltiles, nslabs), dim3(256), 0, stream, X, n, L, CB, slab, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(colsum_final_kernel, dim3((L + 255) / 256), dim3(256), 0, stream, part, nslabs, L, T);
    return hipGetLastError();
}

// Large batches of a matrix that is not sparse enough: the gathers move nnz.4.batch bytes through the L1/L2 path
// (measured 18 - 31 TB/s chip-wide, 24 taken here), the fp32 matrix cores need 2.m.n.batch flops (the dense kernel
// of this library: 12 - 20 us + flops / 90 ... 120 TFLOP/s, rising with the size), so from about one indexed
// element in five upwards the dense contraction is the faster way to the same Y.  The matrix is then decoded into a
// stream-ordered temporary (4.m.n bytes, bounded here; written at about 4.5 TB/s) and multiplied on the matrix
// cores.  Measured on MI355X, gathers against decode + dense: 3x3 convolution shape (60 % zeros) batch 3136
// 391 / 201 us, batch 784 165 / 75 us, batch 256 44 / 45 us; AlexNet-fc6 shape (85 %) batch 2048 1917 / 1466 us,
// batch 512 419 / 421 us; VGG-fc6 shape (95 %) batch 1024 1187 / 2017 us; 2048 x 2048, batch 1024: 70 % zeros
// 187 / 119 us, 80 % 139 / 119 us, 90 % 89 / 118 us.
// Narrow batches of a dense-ish matrix take the same route: a gather moves a whole 128-byte line however narrow the
// batch, so a 4096 x 9216 layer quantized to 7 bits (71 % of the elements indexed) costs 171 us at batch 32 by
// gathers, 70 us decoded (30 us) and multiplied by the dense kernel (40 us, itself bound by reading the matrix).
// Estimated durations (seconds) of the gathers and of decode + dense; false where the dense route is not available.
bool densify_estimates(const DeviceView& d, uint32_t L, double* t_gather_out, double* t_dense_out) {
    if (L < 2 || d.m < 128 || d.n < 256) return false;
    const double mn = (double)d.m * (double)d.n;
    if (mn * 4.0 > (double)(1ull << 30)) return false;
    const double flops = 2.0 * mn * L;
    // every (row, tile) is a wave whose start-up chain (descriptor -> pointers -> indices -> first gathers) takes about
    // 4 us, 4096 of them in flight: what bounds matrices of many short rows (16384 x 512: batch 128 64 - 84 us,
    // batch 512 160 - 440 us by gathers; 44 - 49 us and 94 - 103 us decoded and multiplied)
    const double tiles = std::ceil((double)L / 32.0);
    const double t_gather = std::max((double)d.nnz * std::max(4.0 * L, 128.0) / 24e12, (double)d.m * tiles * 4e-6 / 4096.0);
    const double rate = flops < 1.5e10 ? 90e12 : (flops < 1e11 ? 105e12 : 120e12);
    const double t_write = 4.0 * mn / 4.5e12;  // the decoded matrix goes to memory once and is read back at least once
    const double t_decode = t_write + (double)d.nnz * 1.5e-12 + 3e-6;  // measured 30 us (5.7 M indices) ... 88 us (28.7 M)
    const double t_dense = (flops < 5e9 ? 20e-6 : 12e-6) + std::max(flops / rate, t_write) + t_decode;
    *t_gather_out = t_gather;
    *t_dense_out = t_dense;
    return true;
}

bool densify_pays(const DeviceView& d, uint32_t L) {
    double t_gather = 0, t_dense = 0;
    return densify_estimates(d, L, &t_gather, &t_dense) && t_gather > 1.1 * t_dense;
}

hipError_t launch_densified(const DeviceView& d, const float* X, float* Y, uint32_t L, hipStream_t stream) {
    float* W = nullptr;
    hipError_t e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&W), (size_t)d.m * (size_t)d.n * sizeof(float), stream);
    if (e != hipSuccess) return e;
    if (decode_device(d, W, stream) != 0) e = hipErrorLaunchFailure;  // a CER_* code: only a failed launch is possible
    if (e == hipSuccess) e = (hipError_t)launch_dense(W, X, Y, d.m, d.n, (int64_t)L, stream);
    const hipError_t f = (hipError_t)temp_free(W, stream);
    return e == hipSuccess ? f : e;
}

// Whether the LDS variant is expected to beat the kernel that gathers from L2.  Measured on MI355X: for wide
// batches it never does -- gathers of 16- or 32-byte pieces at random LDS addresses are bank-conflict bound at
// 32 - 43 B/clk per CU, while the L2 kernel's gathers of whole 128-byte rows sustain 27 - 48 B/clk per CU and
// amortise the group structure over 32 batch columns instead of 4 or 8 (AlexNet-fc6 shape, batch 32: 62 us against
// 35 us; 3x3 convolution shape, batch 3136: 536 us against 378 us).  For narrow batches it does: the L2 kernel
// still moves a whole 128-byte line per index, the LDS kernel 16 or 32 bytes (AlexNet-fc6 shape, batch 2 / 3 / 4 /
// 6 / 8: 28 / 29 / 29 / 37 / 31 us from L2, 23 / 22 / 13 / 28 / 28 us from LDS with the tile-major copy, less
// without it), provided the matrix is large enough for the gathers to dominate the launch (2048 x 2048 cells with
// 0.2 - 2 million indices: 6 - 12 us either way, the L2 kernel ahead).
bool xtile_pays(const DeviceView& d, uint32_t L) { return L <= 8 && d.nnz >= 2500000; }

// Which kernel serves a batch of L > 1 columns (cer_matmul_path's numbering: 1, 2 or 3).  A preferred kernel is
// taken whenever it is applicable; otherwise the estimates decide.  no_temporaries: only kernels that need no
// temporary memory (the decode + dense route and batches of more than one LDS tile are left out).
int choose_batched_path(const DeviceView& d, uint32_t L, const MatmulOptions& o, bool no_temporaries, XtilePlan* plan_out,
                        const float* X = nullptr, const float* Y = nullptr) {
    const bool has_elements = d.m > 0 && d.n > 0;
    // strips of X in LDS: on request (and only when the strip-major index was prepared); the partial sums of the strips
    // need a temporary.  X == nullptr: the question is asked without buffers (cer_matmul_path_ex): aligned ones assumed.
    const bool strips_ok = !no_temporaries && strip_applicable(d, X, Y, L);
    if (o.path == kPathStrip && strips_ok) return kPathStrip;
    if (o.path == 3 && has_elements && !no_temporaries) return 3;
    // the strips' estimate against the gathers' (and, below, against decode + dense)
    bool strips_beat_gathers = false;
    double t_strip = 0;
    if (o.path < 0 && strips_ok && has_elements) {
        t_strip = plan_strip(d, L).est_us * 1e-6;
        // bytes a gather moves per index: whole 128-byte lines; a width that is not a multiple of 32 columns touches
        // about one line more per row of X (AlexNet-fc6 shape batch 100: 114 us, VGG-fc6 shape: 158 us), unless a row
        // of X divides a line (8 and 16 columns)
        const double lines = L % 32u == 0 ? L / 32.0 : (L < 32u && 32u % L == 0 ? 1.0 : 0.85 * ((L + 31u) / 32u + 1.0));
        const double t_gather_l2 = 5e-6 + (double)d.nnz * 128.0 * lines / 27e12;
        strips_beat_gathers = t_strip < 0.95 * t_gather_l2;
    }
    // (from 8 columns on the strips are ahead of the LDS tile of all input rows: AlexNet-fc6 shape batch 8 23 against 28 us)
    if (o.path != 1 && o.path != 3 && !(strips_beat_gathers && L >= 8u)) {
        const XtilePlan plan = plan_xtile(d, L);
        if (plan.valid && (o.path == 2 || xtile_pays(d, L)) && (!no_temporaries || plan.ntiles == 1)) {
            if (plan_out) *plan_out = plan;
            return 2;
        }
    }
    // A handle whose strip-major index was prepared takes the strip kernel where its estimate beats that of the
    // gathers from L2 (27 TB/s of whole 128-byte lines plus the start-up chain of a launch) and that of decode +
    // dense: wide batches of large matrices -- AlexNet-fc6 shape, batch 32 / 64 / 128: 25 / 38 / 61 us against
    // 33 / 57 / 107 us; VGG-fc6 shape, batch 64 / 128: 45 / 78 against 54 / 100 us (batch 32: 29 against 31 us: the
    // estimate keeps the gathers; 3x3 convolution shape, batch 3136: 209 us against 159 us decoded and multiplied); batch widths
    // that are multiples of 4 but not of 32: AlexNet-fc6 shape batch 100: 61 against 114 us; batches of 8 - 16 columns
    // (one 16-byte piece of a row per lane): AlexNet-fc6 shape batch 16 20 against 31 us, VGG-fc6 shape 22 against 28 us.
    if (o.path < 0 && !no_temporaries && has_elements) {
        double t_gather = 0, t_dense = 0;
        const bool dense_ok = densify_estimates(d, L, &t_gather, &t_dense);
        const bool dense_pays = dense_ok && t_gather > 1.1 * t_dense;
        if (strips_beat_gathers && (!dense_pays || t_strip < t_dense)) return kPathStrip;
        if (dense_pays) return 3;
    }
    return 1;
}

// Column sums of X for a non-zero most frequent value: shape of the two-stage sum and the floats it needs
// ([T: L rounded to 64][partials: nslabs x L]).
struct ColsumPlan {
    uint32_t CB = 1, nslabs = 1, slab = 1;
    size_t t_floats = 0, floats = 0;
};

// Slabs of 32 rows or more, up to 4096 workgroups: a pass over a large X is bound by how many loads are in flight (3x3
// convolution shape, batch 3136, 58 MB of X: 48 us with slabs of 256 rows).  Where that many partial sums would not fit
// the fixed workspace of the entry point that allocates nothing, slabs of 256 rows and up to 1024 workgroups: both
// entry points sum in the same order.
ColsumPlan plan_colsum(uint32_t n, uint32_t L) {
    ColsumPlan p;
    p.CB = std::min<uint32_t>(256u, pow2_ceil(L));
    const uint32_t coltiles = (L + p.CB - 1) / p.CB;
    p.t_floats = ((size_t)L + 63) & ~(size_t)63;
    for (int wide = 1; wide >= 0; --wide) {
        const uint32_t rows = wide ? 32u : 256u, blocks = wide ? 4096u : 1024u;
        p.nslabs = std::max<uint32_t>(1u, std::min<uint32_t>((n + rows - 1u) / rows, blocks / std::max(coltiles, 1u)));
        p.slab = std::max<uint32_t>((n + p.nslabs - 1) / p.nslabs, 1u);
        p.floats = p.t_floats + (size_t)p.nslabs * L;
        if (p.floats <= kStaticWorkspaceFloats) break;
    }
    return p;
}

}  // namespace

int matmul_path(const DeviceView& d, int64_t L, const MatmulOptions& o) {
    if (L <= 1) return gemv_path(d, o);
    if (L > 0x7FFFFFFFll) return 1;
    return choose_batched_path(d, (uint32_t)L, o, false, nullptr);
}

size_t matmul_workspace_floats(const DeviceView& d, int64_t L, const MatmulOptions& o) {
    if (d.m == 0 || L < 1 || L > 0x7FFFFFFFll || d.omega0 == 0.f) return 0;
    if (L == 1 && gemv_sums_x(d, o)) return 0;
    return plan_colsum((uint32_t)d.n, (uint32_t)L).floats;
}

int static_workspace(float** ptr, size_t* floats) {
    static std::mutex mu;
    static float* addr[16] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= 16) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        addr[dev] = static_cast<float*>(p);
    }
    *ptr = addr[dev];
    *floats = kStaticWorkspaceFloats;
    return (int)hipSuccess;
}

int launch_matmul(const DeviceView& d, const float* X, float* Y, int64_t L64, void* stream_v, const MatmulOptions& o_in,
                  float* workspace, size_t workspace_floats) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (d.m == 0) return (int)hipSuccess;
    if (L64 > 0x7FFFFFFFll || d.m > 0x7FFFFFFFll) return (int)hipErrorInvalidValue;
    const uint32_t L = (uint32_t)L64;
    const bool no_temporaries = workspace != nullptr;
    MatmulOptions o = o_in;
    if (no_temporaries) o.flags |= kOptRowsWhole;  // the parts of split rows meet in a temporary
    XtilePlan plan;
    const int batched_path = L > 1 ? choose_batched_path(d, L, o, no_temporaries, &plan, X, Y) : 0;
    if (batched_path == 3) return (int)launch_densified(d, X, Y, L, stream);

    float* T = nullptr;
    float* scratch = nullptr;
    hipError_t e = hipSuccess;
    if (d.omega0 != 0.f && !(L == 1 && gemv_sums_x(d, o))) {
        // T[l] = sum_i X[i,l], in the caller's workspace or in a stream-ordered temporary
        const ColsumPlan cp = plan_colsum((uint32_t)d.n, L);
        float* base = workspace;
        if (no_temporaries) {
            if (cp.floats > workspace_floats) return (int)hipErrorInvalidValue;  // the caller has checked the size
        } else {
            e = (hipError_t)temp_alloc(reinterpret_cast<void**>(&scratch), cp.floats * sizeof(float), stream);
            if (e != hipSuccess) return (int)e;
            base = scratch;
        }
        T = base;
        e = launch_colsum(X, (uint32_t)d.n, L, base + cp.t_floats, cp.nslabs, cp.slab, cp.CB, T, stream);
        if (e != hipSuccess) {
            if (scratch) (void)temp_free(scratch, stream);
            return (int)e;
        }
    }
    if (L == 1)
        e = launch_gemv_any(d, X, Y, T, stream, o);
    else if (batched_path == 2)
        e = launch_xtile_any(d, plan, X, Y, T, L, stream);
    else if (batched_path == kPathStrip)
        e = launch_strip(d, X, Y, T, L, stream);
    else
        e = launch_gemm_any(d, X, Y, T, L, stream, o);
    if (scratch) {
        hipError_t f = (hipError_t)temp_free(scratch, stream);
        if (e == hipSuccess) e = f;
    }
    return (int)e;
}

}  // namespace cer
