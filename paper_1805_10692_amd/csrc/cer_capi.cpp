// extern "C" boundary of the library: argument checks, handle lifetime, device upload.
#include <algorithm>
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "../../include/cer.h"
#include "cer_internal.hpp"

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return CER_E_HIP;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int cer::record_hip_error(int hip_error) {
    g_last_hip_error = hip_error;
    return CER_E_HIP;
}

// ---- stream-ordered temporaries from a pool of the library's own ------------------------------------------------
namespace {
struct TempPool {
    std::mutex mu;
    bool tried = false;
    hipMemPool_t pool = nullptr;  // nullptr after a failed creation: the device's default pool serves instead
};
TempPool g_temp_pools[16];

// The library's pool on the current device, created on first use.
hipMemPool_t temp_pool() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    TempPool& t = g_temp_pools[dev];
    std::lock_guard<std::mutex> lock(t.mu);
    if (!t.tried) {
        t.tried = true;
        hipMemPoolProps props;
        std::memset(&props, 0, sizeof props);
        props.allocType = hipMemAllocationTypePinned;
        props.handleTypes = hipMemHandleTypeNone;
        props.location.type = hipMemLocationTypeDevice;
        props.location.id = dev;
        hipMemPool_t pool = nullptr;
        if (hipMemPoolCreate(&pool, &props) == hipSuccess) {
            uint64_t keep = UINT64_MAX;  // nothing goes back to the system before cer_trim
            if (hipMemPoolSetAttribute(pool, hipMemPoolAttrReleaseThreshold, &keep) == hipSuccess)
                t.pool = pool;
            else
                (void)hipMemPoolDestroy(pool);
        }
        (void)hipGetLastError();  // a failed creation is not an error of the call that asked for memory
    }
    return t.pool;
}
}  // namespace

int cer::temp_alloc(void** p, size_t bytes, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipMemPool_t pool = temp_pool();
    return (int)(pool ? hipMallocFromPoolAsync(p, bytes, pool, s) : hipMallocAsync(p, bytes, s));
}

int cer::temp_free(void* p, void* stream) { return (int)hipFreeAsync(p, static_cast<hipStream_t>(stream)); }


namespace {

std::vector<uint32_t> widen(const cer::HostArray& a) {
    std::vector<uint32_t> out((size_t)a.len);
    for (int64_t i = 0; i < a.len; ++i) out[(size_t)i] = (uint32_t)a.at(i);
    return out;
}

}  // namespace

cer::DeviceLayout cer::DeviceLayout::make(size_t colI_bytes, int64_t G, int64_t m, size_t omegaI_bytes, int32_t K) {
    DeviceLayout l;
    l.colI_bytes = colI_bytes;
    l.omegaI_bytes = omegaI_bytes;
    l.off_colI = 0;
    l.off_optr = align_up(l.off_colI + colI_bytes + 8192, 256);  // the product reads ahead of a row's end
    l.off_rptr = align_up(l.off_optr + (size_t)(G + 1) * 4 + 16, 256);
    l.off_oi = align_up(l.off_rptr + (size_t)(m + 1) * 4 + 16, 256);
    l.off_om = align_up(l.off_oi + omegaI_bytes + 16, 256);
    l.off_ri = align_up(l.off_om + (size_t)std::max(K, 1) * 4, 256);
    l.off_tab = align_up(l.off_ri + (size_t)(m + 1) * 8, 256);
    size_t tab_bytes = 0;
    if (K >= 2 && K <= 256 && m > 0) {  // rank table: 4 .. 256 words per row
        l.tab_shift = 2;
        while ((1 << l.tab_shift) < K) ++l.tab_shift;
        tab_bytes = ((size_t)m << l.tab_shift) * 4 + 256;
    }
    l.total = align_up(l.off_tab + tab_bytes, 256);
    return l;
}

namespace {
// Compute units and LDS per workgroup of a device, read once per device.
struct DeviceProps {
    std::once_flag once;
    int cus = 256;
    size_t lds_per_block = 64 * 1024;
};
DeviceProps g_device_props[16];

const DeviceProps& device_props(int dev) {
    DeviceProps& p = g_device_props[(dev >= 0 && dev < 16) ? dev : 0];
    std::call_once(p.once, [&p, dev] {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            p.cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
            p.lds_per_block = std::max<size_t>(prop.sharedMemPerBlock, prop.maxSharedMemoryPerMultiProcessor);
        } else {
            (void)hipGetLastError();
        }
    });
    return p;
}
}  // namespace

void cer::bind_device(cer_matrix* h, int dev, void* base, const DeviceLayout& l) {
    const HostMatrix& A = *h->host;
    auto* b = static_cast<unsigned char*>(base);
    h->device = dev;
    h->d_base = base;
    h->d_bytes = l.total;
    h->stream_bytes = (int64_t)(l.colI_bytes + (size_t)(A.G + 1) * 4 + (size_t)(A.m + 1) * 4 + l.omegaI_bytes +
                                A.omega.size() * 4);
    DeviceView& v = h->view;
    v.colI = b + l.off_colI;
    v.omegaPtr = reinterpret_cast<const uint32_t*>(b + l.off_optr);
    v.rowPtr = reinterpret_cast<const uint32_t*>(b + l.off_rptr);
    v.omegaI = b + l.off_oi;
    v.omega = reinterpret_cast<const float*>(b + l.off_om);
    v.rowInfo = b + l.off_ri;
    v.rank_tab = l.tab_shift ? reinterpret_cast<const uint32_t*>(b + l.off_tab) : nullptr;
    v.rank_tab_shift = l.tab_shift;
    v.colI_bits = A.colI.bits;
    v.omegaI_bits = A.omegaI.bits;
    v.cser = A.cser ? 1 : 0;
    v.K = A.K;
    v.m = A.m;
    v.n = A.n;
    v.max_row_groups = A.max_row_groups;
    v.nnz = A.nnz;
    v.nonempty_groups = A.nonempty_groups;
    v.omega0 = A.K > 0 ? A.omega[0] : 0.f;
    const DeviceProps& dp = device_props(dev);
    v.cus = dp.cus;
    v.lds_per_block = dp.lds_per_block;
    h->layout = l;
}

int cer::ensure_host_arrays(const cer_matrix* h) {
    const HostMatrix& A = *h->host;
    if (A.arrays_on_host.load(std::memory_order_acquire)) return CER_OK;
    std::lock_guard<std::mutex> lock(A.fetch_mutex);
    if (A.arrays_on_host.load(std::memory_order_relaxed)) return CER_OK;
    if (h->device < 0 || !h->d_base) return CER_E_INVALID;
    const auto* b = static_cast<const unsigned char*>(h->d_base);
    const DeviceLayout& l = h->layout;
    hipError_t e = hipSuccess;
    auto get = [&](void* dst, size_t off, size_t bytes) {
        if (e == hipSuccess && bytes) e = hipMemcpy(dst, b + off, bytes, hipMemcpyDeviceToHost);
    };
    auto narrow = [](const std::vector<uint32_t>& src, HostArray& dst) {  // dst.len and dst.bits are already set
        dst.bytes.resize(src.size() * (size_t)(dst.bits / 8));
        for (size_t i = 0; i < src.size(); ++i) {
            if (dst.bits == 8) dst.bytes[i] = (uint8_t)src[i];
            else if (dst.bits == 16) reinterpret_cast<uint16_t*>(dst.bytes.data())[i] = (uint16_t)src[i];
            else reinterpret_cast<uint32_t*>(dst.bytes.data())[i] = src[i];
        }
    };
    A.colI.bytes.resize(l.colI_bytes);
    get(A.colI.bytes.data(), l.off_colI, l.colI_bytes);
    A.omegaI.bytes.resize(l.omegaI_bytes);
    get(A.omegaI.bytes.data(), l.off_oi, l.omegaI_bytes);
    std::vector<uint32_t> optr((size_t)A.G + 1), rptr((size_t)A.m + 1);
    get(optr.data(), l.off_optr, optr.size() * 4);
    get(rptr.data(), l.off_rptr, rptr.size() * 4);
    if (e != hipSuccess) return hip_fail(e);
    narrow(optr, A.omegaPtr);
    narrow(rptr, A.rowPtr);
    A.arrays_on_host.store(true, std::memory_order_release);
    return CER_OK;
}

namespace {

// The row schedule of a host-encoded handle, from its host arrays.
int upload_split_table(cer_matrix* h) {
    const cer::HostMatrix& A = *h->host;
    if (A.m <= 0 || A.nnz <= 0) return CER_OK;
    std::vector<uint64_t> start((size_t)A.m + 1);
    for (int64_t r = 0; r <= A.m; ++r) start[(size_t)r] = A.omegaPtr.at((int64_t)A.rowPtr.at(r));
    return cer::build_row_schedule(h, start);
}

}  // namespace

namespace {
// P: positions per part of a long row
uint64_t part_length(uint64_t mean) { return ((std::max<uint64_t>(mean + mean / 2, 2048) + 2047) / 2048) * 2048; }
}  // namespace

bool cer::row_schedule_wanted(uint64_t nnz, uint64_t m, uint64_t longest) {
    if (m == 0 || nnz == 0) return false;
    const uint64_t mean = nnz / m;
    if (longest < 2048 || longest <= 2 * mean) return false;
    // rows of a few dozen indices are bound by their wave's start-up chain, to which the look-up of the row adds a
    // step: 16384 x 4096 with 41 indices per row and three rows of about 3000 measured 8 % slower in order
    return mean >= 256 || longest > 3 * part_length(mean);
}

// Rows of unequal length (pruned layers; matrices of independent elements have none).  One wave serves one row per
// batch tile and a workgroup holds its resources until its longest row is done, so the batched product
//  - takes the rows in descending order of length when the longest row holds more than twice the average (and at
//    least 2048 positions; the average row at least 256, or some row is split): the four rows of a workgroup are
//    then about equally long and the long rows start first;
//  - serves rows in parts when one of them would outlast the launch: if some row holds more than 3 P positions, P =
//    1.5 x the average row rounded up to a multiple of 2048, the rows of more than 2 P positions are split into parts
//    of P positions (the table lists every part but a row's first; the second kernel and the temporary that the parts
//    need cost about 6 us per product, hence the 3 P).
// Device table: [order: m x uint32][parts: {row, first position, end position, 0}][rows: {row, first part, parts, 0}].
int cer::build_row_schedule(cer_matrix* h, const std::vector<uint64_t>& start) {
    const cer::HostMatrix& A = *h->host;
    if (A.m <= 0 || A.nnz <= 0 || h->device < 0) return CER_OK;
    uint64_t longest = 0;
    for (int64_t r = 0; r < A.m; ++r) longest = std::max(longest, start[(size_t)r + 1] - start[(size_t)r]);
    if (!row_schedule_wanted((uint64_t)A.nnz, (uint64_t)A.m, longest)) return CER_OK;
    const uint64_t mean = (uint64_t)(A.nnz / A.m);
    const uint64_t len = part_length(mean);

    std::vector<uint32_t> order((size_t)A.m);
    for (int64_t r = 0; r < A.m; ++r) order[(size_t)r] = (uint32_t)r;
    std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        return start[(size_t)a + 1] - start[a] > start[(size_t)b + 1] - start[b];
    });

    std::vector<uint32_t> parts, rows;
    if (longest > 3 * len && len <= 0x3FFFFFFFull) {
        for (int64_t r = 0; r < A.m; ++r) {
            const uint64_t rs = start[(size_t)r], re = start[(size_t)r + 1];
            if (re - rs <= 2 * len) continue;
            const uint32_t first = (uint32_t)(parts.size() / 4);
            for (uint64_t b = rs + len; b < re; b += len) {
                parts.push_back((uint32_t)r);
                parts.push_back((uint32_t)b);
                parts.push_back((uint32_t)std::min(re, b + len));
                parts.push_back(0u);
            }
            rows.push_back((uint32_t)r);
            rows.push_back(first);
            rows.push_back((uint32_t)(parts.size() / 4) - first);
            rows.push_back(0u);
        }
    }
    const size_t order_bytes = (order.size() * 4 + 15) & ~(size_t)15, part_bytes = parts.size() * 4, row_bytes = rows.size() * 4;
    void* base = nullptr;
    hipError_t e = hipMalloc(&base, order_bytes + part_bytes + row_bytes + 16);
    if (e != hipSuccess) return hip_fail(e);
    auto* b8 = static_cast<unsigned char*>(base);
    e = hipMemcpy(b8, order.data(), order.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess && part_bytes) e = hipMemcpy(b8 + order_bytes, parts.data(), part_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess && row_bytes) e = hipMemcpy(b8 + order_bytes + part_bytes, rows.data(), row_bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(e);
    }
    h->d_split = base;
    h->view.row_order = base;
    h->view.split_parts = b8 + order_bytes;
    h->view.split_rows = b8 + order_bytes + part_bytes;
    h->view.n_split_parts = (uint32_t)(parts.size() / 4);
    h->view.n_split_rows = (uint32_t)(rows.size() / 4);
    h->view.split_len = (uint32_t)len;
    h->view.split_min = parts.empty() ? 0xFFFFFFFFu : (uint32_t)(2 * len);
    return CER_OK;
}

namespace {

// Copies the host arrays into one fresh device allocation (layout: cer::DeviceLayout).
int upload(cer_matrix* h) {
    const cer::HostMatrix& A = *h->host;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        h->device = -1;
        return CER_OK;  // host-only handle
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);

    const cer::DeviceLayout l = cer::DeviceLayout::make(A.colI.bytes.size(), A.G, A.m, A.omegaI.bytes.size(), A.K);
    void* base = nullptr;
    e = hipMalloc(&base, l.total);
    if (e != hipSuccess) return hip_fail(e);
    auto* b = static_cast<unsigned char*>(base);
    e = hipMemset(base, 0, l.total);
    auto put = [&](size_t off, const void* src, size_t bytes) {
        if (e == hipSuccess && bytes) e = hipMemcpy(b + off, src, bytes, hipMemcpyHostToDevice);
    };
    put(l.off_colI, A.colI.bytes.data(), l.colI_bytes);
    {
        std::vector<uint32_t> w = widen(A.omegaPtr);
        put(l.off_optr, w.data(), w.size() * 4);
    }
    {
        std::vector<uint32_t> w = widen(A.rowPtr);
        put(l.off_rptr, w.data(), w.size() * 4);
        std::vector<uint32_t> info((size_t)(A.m + 1) * 2);
        for (int64_t r = 0; r <= A.m; ++r) {
            info[(size_t)r * 2] = w[(size_t)r];
            info[(size_t)r * 2 + 1] = (uint32_t)A.omegaPtr.at((int64_t)w[(size_t)r]);
        }
        put(l.off_ri, info.data(), info.size() * 4);
    }
    put(l.off_oi, A.omegaI.bytes.data(), l.omegaI_bytes);
    put(l.off_om, A.omega.data(), A.omega.size() * 4);
    if (e != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(e);
    }
    cer::bind_device(h, dev, base, l);
    e = (hipError_t)cer::build_rank_table(h->view, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) return hip_fail(e);  // the caller frees the handle and with it the allocation
    return upload_split_table(h);
}

int encode_any(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, bool cser, cer_handle_t** out) {
    if (!out) return CER_E_INVALID;
    *out = nullptr;
    if (m < 0 || n < 0 || K < 0) return CER_E_INVALID;
    if ((m > 0 && n > 0 && !W) || (K > 0 && !codebook)) return CER_E_INVALID;
    if (m > 0 && n > 0 && K == 0) return CER_E_NOT_IN_CODEBOOK;
    if (m > 0x7FFFFFFFll) return CER_E_TOO_LARGE;
    try {
        std::shared_ptr<cer::HostMatrix> host;
        int rc = cer::encode_host(W, m, n, codebook, K, cser, &host);
        if (rc != CER_OK) return rc;
        auto* h = new cer_matrix();
        h->host = std::move(host);
        rc = upload(h);
        if (rc != CER_OK) {
            cer_free(h);
            return rc;
        }
        *out = h;
        return CER_OK;
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    } catch (...) {
        return CER_E_INVALID;
    }
}

// cer_matmul_opts_t -> the launchers' options; false: a field holds a value the header does not define.
bool read_options(const cer_matmul_opts_t* in, cer::MatmulOptions* out) {
    *out = cer::MatmulOptions{};
    if (!in) return true;
    constexpr uint32_t known = CER_OPT_SUM_THEN_MULTIPLY | CER_OPT_ROWS_WHOLE | CER_OPT_X_FROM_GLOBAL |
                               CER_OPT_ONE_COLUMN_PER_LANE | CER_OPT_SHORT_CHUNKS | CER_OPT_LONG_CHUNKS |
                               CER_OPT_NO_RANK_TABLE;
    if (in->path < CER_PATH_AUTO || in->path > CER_PATH_STRIP) return false;
    if (in->flags & ~known) return false;
    if ((in->flags & CER_OPT_SHORT_CHUNKS) && (in->flags & CER_OPT_LONG_CHUNKS)) return false;
    switch (in->tile_cols) {
        case 0: case 8: case 16: case 32: case 64: case 128: break;
        default: return false;
    }
    out->path = in->path;
    out->tile_cols = in->tile_cols;
    out->flags = in->flags;
    return true;
}

// The handle's device is the current one and holds its arrays; else the CER_* code to return.
int check_device(const cer_handle_t* h) {
    if (h->device < 0 || !h->d_base) {
        g_last_hip_error = (int)hipErrorNoDevice;
        return CER_E_HIP;
    }
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev != h->device) return hip_fail(hipErrorInvalidDevice);
    return CER_OK;
}

int matmul_any(const cer_handle_t* h, int want_cser /* -1: either */, const float* X, float* Y, int64_t batch, void* stream,
               const cer_matmul_opts_t* opts) {
    if (!h || !X || !Y || batch < 1) return CER_E_INVALID;
    if (want_cser >= 0 && h->host->cser != (want_cser != 0)) return CER_E_FORMAT;
    cer::MatmulOptions o;
    if (!read_options(opts, &o)) return CER_E_INVALID;
    const int dc = check_device(h);
    if (dc != CER_OK) return dc;
    const int rc = cer::launch_matmul(h->view, X, Y, batch, stream, o);
    return rc == 0 ? CER_OK : hip_fail((hipError_t)rc);
}

int decode_any(const cer_handle_t* h, bool want_cser, float* W_out) {
    if (!h) return CER_E_INVALID;
    if (h->host->cser != want_cser) return CER_E_FORMAT;
    if (!W_out && h->host->m * h->host->n > 0) return CER_E_INVALID;
    try {
        const int rc = cer::ensure_host_arrays(h);
        if (rc != CER_OK) return rc;
        return cer::decode_host(*h->host, W_out);
    } catch (...) {
        return CER_E_NOMEM;
    }
}

}  // namespace

extern "C" {

int cer_encode(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, cer_handle_t** out) {
    return encode_any(W, m, n, codebook, K, false, out);
}
int cser_encode(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, cer_handle_t** out) {
    return encode_any(W, m, n, codebook, K, true, out);
}

int cer_matmul(const cer_handle_t* h, const float* X, float* Y, int64_t batch, void* stream) {
    return matmul_any(h, 0, X, Y, batch, stream, nullptr);
}
int cser_matmul(const cer_handle_t* h, const float* X, float* Y, int64_t batch, void* stream) {
    return matmul_any(h, 1, X, Y, batch, stream, nullptr);
}
int cer_matmul_ex(const cer_handle_t* h, const float* X, float* Y, int64_t batch, void* stream,
                  const cer_matmul_opts_t* opts) {
    return matmul_any(h, -1, X, Y, batch, stream, opts);
}

int cer_matmul_noalloc(const cer_handle_t* h, const float* X, float* Y, int64_t batch, void* stream) {
    if (!h || !X || !Y || batch < 1) return CER_E_INVALID;
    const int dc = check_device(h);
    if (dc != CER_OK) return dc;
    float* ws = nullptr;
    size_t ws_floats = 0;
    const int we = cer::static_workspace(&ws, &ws_floats);
    if (we != 0) return hip_fail((hipError_t)we);
    const cer::MatmulOptions o;
    if (cer::matmul_workspace_floats(h->view, batch, o) > ws_floats) return CER_E_TOO_LARGE;
    const int rc = cer::launch_matmul(h->view, X, Y, batch, stream, o, ws, ws_floats);
    return rc == 0 ? CER_OK : hip_fail((hipError_t)rc);
}

int cer_matmul_path_ex(const cer_handle_t* h, int64_t batch, const cer_matmul_opts_t* opts) {
    if (!h || batch < 1) return CER_E_INVALID;
    cer::MatmulOptions o;
    if (!read_options(opts, &o)) return CER_E_INVALID;
    if (h->device < 0 || !h->d_base) return CER_E_HIP;
    return cer::matmul_path(h->view, batch, o);
}
int cer_matmul_path(const cer_handle_t* h, int64_t batch) { return cer_matmul_path_ex(h, batch, nullptr); }

int cer_decode(const cer_handle_t* h, float* W_out) { return decode_any(h, false, W_out); }
int cser_decode(const cer_handle_t* h, float* W_out) { return decode_any(h, true, W_out); }

int cer_get_array(const cer_handle_t* h, int which, const void** host_ptr, int64_t* len, int32_t* elem_bits) {
    if (!h || !host_ptr || !len || !elem_bits) return CER_E_INVALID;
    const cer::HostMatrix& A = *h->host;
    const cer::HostArray* a = nullptr;
    switch (which) {
        case CER_ARRAY_OMEGA: *host_ptr = A.omega.data(); *len = A.K; *elem_bits = 32; return CER_OK;
        case CER_ARRAY_COUNT: *host_ptr = A.count.data(); *len = A.K; *elem_bits = 64; return CER_OK;
        case CER_ARRAY_COLI: a = &A.colI; break;
        case CER_ARRAY_OMEGAPTR: a = &A.omegaPtr; break;
        case CER_ARRAY_ROWPTR: a = &A.rowPtr; break;
        case CER_ARRAY_OMEGAI: a = &A.omegaI; break;
        default: return CER_E_INVALID;
    }
    try {
        const int rc = cer::ensure_host_arrays(h);
        if (rc != CER_OK) return rc;
    } catch (...) {
        return CER_E_NOMEM;
    }
    *host_ptr = a->bytes.data();
    *len = a->len;
    *elem_bits = a->bits;
    return CER_OK;
}

int cer_get_dims(const cer_handle_t* h, int64_t* m, int64_t* n, int32_t* K, int64_t* nnz, int64_t* groups,
                 int32_t* is_cser) {
    if (!h) return CER_E_INVALID;
    const cer::HostMatrix& A = *h->host;
    if (m) *m = A.m;
    if (n) *n = A.n;
    if (K) *K = A.K;
    if (nnz) *nnz = A.nnz;
    if (groups) *groups = A.G;
    if (is_cser) *is_cser = A.cser ? 1 : 0;
    return CER_OK;
}

int64_t cer_storage_bits(const cer_handle_t* h) {
    if (!h) return CER_E_INVALID;
    const cer::HostMatrix& A = *h->host;
    int64_t bits = (int64_t)A.K * 32 + A.colI.len * A.colI.bits + A.omegaPtr.len * A.omegaPtr.bits +
                   A.rowPtr.len * A.rowPtr.bits;
    if (A.cser) bits += A.omegaI.len * A.omegaI.bits;
    return bits;
}

int cer_get_stats(const cer_handle_t* h, double* H, double* p0, double* k_bar, double* k_tilde) {
    if (!h) return CER_E_INVALID;
    const cer::HostMatrix& A = *h->host;
    const double N = (double)A.m * (double)A.n;
    double ent = 0.0;
    for (int32_t k = 0; k < A.K; ++k) {
        const double p = N > 0 ? (double)A.count[(size_t)k] / N : 0.0;
        if (p > 0) ent -= p * std::log2(p);
    }
    if (H) *H = ent;
    if (p0) *p0 = (A.K > 0 && N > 0) ? (double)A.count[0] / N : 0.0;
    if (k_bar) *k_bar = A.m > 0 ? (double)A.nonempty_groups / (double)A.m : 0.0;
    if (k_tilde) *k_tilde = A.m > 0 ? (double)(A.G - A.nonempty_groups) / (double)A.m : 0.0;
    return CER_OK;
}

int cer_clone_device(const cer_handle_t* h, cer_handle_t** out) {
    if (!h || !out) return CER_E_INVALID;
    *out = nullptr;
    try {
        int rc = cer::ensure_host_arrays(h);
        if (rc != CER_OK) return rc;
        auto* c = new cer_matrix();
        c->host = h->host;
        rc = upload(c);
        if (rc != CER_OK) {
            cer_free(c);
            return rc;
        }
        *out = c;
        return CER_OK;
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    }
}

static int device_front_end(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, int32_t bits,
                            int32_t format, void* stream, float* codebook_out, int32_t* K_out, cer_handle_t** out) {
    if (!out) return CER_E_INVALID;
    *out = nullptr;
    if (K_out) *K_out = 0;
    if (m < 0 || n < 0 || (format != CER_FORMAT_CER && format != CER_FORMAT_CSER)) return CER_E_INVALID;
    if (m > 0 && n > 0 && !W) return CER_E_INVALID;
    if (m > 0x7FFFFFFFll || n > (int64_t)0xFFFFFFFFll) return CER_E_TOO_LARGE;
    const bool cser = format == CER_FORMAT_CSER;
    if (m == 0 || n == 0) return encode_any(nullptr, m, n, codebook, bits > 0 ? 0 : K, cser, out);  // nothing to read
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return hip_fail(hipErrorNoDevice);
    }
    try {
        return cer::encode_device(W, m, n, codebook, K, bits, cser, stream, codebook_out, K_out, out);
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    } catch (...) {
        return CER_E_INVALID;
    }
}

int cer_encode_device(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, int32_t format, void* stream,
                      cer_handle_t** out) {
    if (K < 0 || (K > 0 && !codebook)) return CER_E_INVALID;
    if (K > 256) return CER_E_TOO_LARGE;
    if (m > 0 && n > 0 && K == 0) return CER_E_NOT_IN_CODEBOOK;
    return device_front_end(W, m, n, codebook, K, 0, format, stream, nullptr, nullptr, out);
}

int cer_quantize_encode_device(const float* W, int64_t m, int64_t n, int32_t bits, int32_t format, void* stream,
                               float* codebook_out, int32_t* K_out, cer_handle_t** out) {
    if (bits < 1 || bits > 8) return CER_E_INVALID;
    return device_front_end(W, m, n, nullptr, 0, bits, format, stream, codebook_out, K_out, out);
}

int cer_decode_device(const cer_handle_t* h, float* W, void* stream) {
    if (!h) return CER_E_INVALID;
    if (!W && h->host->m * h->host->n > 0) return CER_E_INVALID;
    if (h->device < 0 || !h->d_base) return hip_fail(hipErrorNoDevice);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev != h->device) return hip_fail(hipErrorInvalidDevice);
    if (h->host->m * h->host->n > 0 && h->host->K < 1) return CER_E_INVALID;
    return cer::decode_device(h->view, W, stream);
}

int cer_quantize_uniform(const float* W, int64_t count, int32_t bits, uint8_t* codes, float* Wq, float* codebook_out,
                         int32_t* K_out, void* stream) {
    if (K_out) *K_out = 0;
    if (bits < 1 || bits > 8 || count < 0 || (count > 0 && !W)) return CER_E_INVALID;
    if (count == 0) return CER_OK;
    if (count > ((int64_t)1 << 42)) return CER_E_TOO_LARGE;
    try {
        return cer::quantize_device(W, count, bits, codes, Wq, codebook_out, K_out, stream);
    } catch (...) {
        return CER_E_NOMEM;
    }
}

int cer_prepare_strips(cer_handle_t* h) {
    if (!h) return CER_E_INVALID;
    if (h->d_strip) return CER_OK;
    const cer::HostMatrix& A = *h->host;
    if (A.K > 64) return CER_E_TOO_LARGE;  // the rank shares 16 bits with the column inside the strip
    if (h->device < 0 || !h->d_base) return hip_fail(hipErrorNoDevice);
    if (A.m <= 0 || A.n <= 0) return CER_OK;
    const int dc = check_device(h);
    if (dc != CER_OK) return dc;
    try {
        const int rc = cer::ensure_host_arrays(h);
        if (rc != CER_OK) return rc;
        // as few strips as 1024 rows each allow, all equally long (4608 columns: five strips of 922, not four of 1024
        // and a half-empty fifth)
        const uint64_t ns = ((uint64_t)A.n + cer::kStripRows - 1) / cer::kStripRows, m = (uint64_t)A.m;
        const uint64_t S = ((uint64_t)A.n + ns - 1) / ns;
        if (ns * (m + 1) > 0x7FFFFFFFull) return CER_E_TOO_LARGE;
        // rank of every raw group (Algorithm 3: position in the row + 1; Algorithm 4: OmegaI)
        std::vector<uint32_t> ptr((size_t)(ns * (m + 1)) + 1, 0u);
        auto for_each = [&](auto&& fn) {
            for (uint64_t r = 0; r < m; ++r) {
                const uint64_t ga = A.rowPtr.at((int64_t)r), gb = A.rowPtr.at((int64_t)r + 1);
                for (uint64_t g = ga; g < gb; ++g) {
                    const uint32_t rank = A.cser ? (uint32_t)A.omegaI.at((int64_t)g) : (uint32_t)(g - ga + 1);
                    const uint64_t pa = A.omegaPtr.at((int64_t)g), pb = A.omegaPtr.at((int64_t)g + 1);
                    for (uint64_t p = pa; p < pb; ++p) fn(r, rank, (uint64_t)A.colI.at((int64_t)p));
                }
            }
        };
        for_each([&](uint64_t r, uint32_t, uint64_t c) { ++ptr[(size_t)((c / S) * (m + 1) + r) + 1]; });
        // entries -> chunks of eight (the last chunk of a (strip, row) is padded with entries of rank 0: weight zero),
        // then counts -> offsets; the entry after each strip's m rows stays a running total, so ptr[s * (m + 1) + m]
        // closes row m - 1
        for (size_t i = 1; i < ptr.size(); ++i) ptr[i] = (ptr[i] + 7u) / 8u;
        for (size_t i = 1; i < ptr.size(); ++i) {
            if ((uint64_t)ptr[i] + ptr[i - 1] >= 0xFFFFFFFFull) return CER_E_TOO_LARGE;
            ptr[i] += ptr[i - 1];
        }
        const uint64_t nchunks = ptr.back();
        std::vector<uint16_t> idx(((size_t)nchunks + 1) * 8, (uint16_t)0);  // one chunk of zeros closes the index
        std::vector<uint64_t> fill(ptr.size() - 1);
        for (size_t i = 0; i + 1 < ptr.size(); ++i) fill[i] = (uint64_t)ptr[i] * 8u;
        for_each([&](uint64_t r, uint32_t rank, uint64_t c) {
            const uint64_t s = c / S;
            idx[(size_t)fill[(size_t)(s * (m + 1) + r)]++] = (uint16_t)((rank << 10) | (uint32_t)(c - s * S));
        });
        const size_t idx_bytes = (idx.size() * 2 + 255) & ~(size_t)255, ptr_bytes = (ptr.size() - 1) * 4;
        void* base = nullptr;
        hipError_t e = hipMalloc(&base, idx_bytes + ptr_bytes + 256);
        if (e != hipSuccess) return hip_fail(e);
        auto* b8 = static_cast<unsigned char*>(base);
        if (!idx.empty()) e = hipMemcpy(b8, idx.data(), idx.size() * 2, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(b8 + idx_bytes, ptr.data(), ptr_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(base);
            return hip_fail(e);
        }
        h->d_strip = base;
        h->view.strip_idx = base;
        h->view.strip_ptr = reinterpret_cast<const uint32_t*>(b8 + idx_bytes);
        h->view.n_strips = (uint32_t)ns;
        h->view.strip_rows = (uint32_t)S;
        h->view.strip_chunks = nchunks;
        return CER_OK;
    } catch (const std::bad_alloc&) {
        return CER_E_NOMEM;
    } catch (...) {
        return CER_E_INVALID;
    }
}

int64_t cer_device_bytes(const cer_handle_t* h) { return (h && h->device >= 0) ? h->stream_bytes : 0; }

int64_t cer_long_row_parts(const cer_handle_t* h) { return (h && h->device >= 0) ? (int64_t)h->view.n_split_parts : 0; }

void cer_free(cer_handle_t* h) {
    if (!h) return;
    if (h->d_base) (void)hipFree(h->d_base);
    if (h->d_split) (void)hipFree(h->d_split);
    if (h->d_strip) (void)hipFree(h->d_strip);
    delete h;
}

int dense_matmul(const float* W, const float* X, float* Y, int64_t m, int64_t n, int64_t batch, void* stream) {
    if (m < 0 || n < 0 || batch < 1) return CER_E_INVALID;
    if (!Y || (n > 0 && m > 0 && !W) || (n > 0 && !X)) return CER_E_INVALID;
    const int rc = cer::launch_dense(W, X, Y, m, n, batch, stream);
    return rc == 0 ? CER_OK : hip_fail((hipError_t)rc);
}

int cer_stream_copy(void* dst, const void* src, int64_t bytes, void* stream) {
    if (!dst || !src || bytes < 0) return CER_E_INVALID;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) return CER_E_INVALID;
    const int rc = cer::launch_stream_copy(dst, src, bytes, stream);
    return rc == 0 ? CER_OK : hip_fail((hipError_t)rc);
}

int cer_stream_read(const void* src, int64_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes < 0) return CER_E_INVALID;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return CER_E_INVALID;
    const int rc = cer::launch_stream_read(src, bytes, sink, stream);
    return rc == 0 ? CER_OK : hip_fail((hipError_t)rc);
}

int cer_trim(void) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hip_fail(hipGetLastError());
    if (dev < 0 || dev >= 16) return CER_OK;
    TempPool& t = g_temp_pools[dev];
    std::lock_guard<std::mutex> lock(t.mu);
    if (!t.pool) return CER_OK;
    const hipError_t e = hipMemPoolTrimTo(t.pool, 0);
    return e == hipSuccess ? CER_OK : hip_fail(e);
}

const char* cer_strerror(int code) {
    switch (code) {
        case CER_OK: return "ok";
        case CER_E_INVALID: return "invalid argument";
        case CER_E_NOT_IN_CODEBOOK: return "matrix element not in codebook";
        case CER_E_BAD_CODEBOOK: return "codebook has a duplicate, NaN or infinite value";
        case CER_E_TOO_LARGE: return "matrix too large for 32-bit indices";
        case CER_E_NOMEM: return "out of host memory";
        case CER_E_HIP: return "HIP error or no device copy";
        case CER_E_FORMAT: return "handle has the other format";
        default: return "unknown error";
    }
}

int cer_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
