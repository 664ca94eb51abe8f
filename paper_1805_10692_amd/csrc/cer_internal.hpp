// Internal declarations shared by the host encoder, the C ABI and the HIP launchers.
#pragma once

#include <atomic>
#include <cstdint>
#include <memory>
#include <mutex>
#include <vector>

struct cer_matrix;

namespace cer {

// One index array of the format, kept on the host at its minimal width (Section V).
struct HostArray {
    std::vector<uint8_t> bytes;
    int64_t len = 0;
    int32_t bits = 8;
    uint64_t at(int64_t i) const {
        switch (bits) {
            case 8: return bytes[(size_t)i];
            case 16: return reinterpret_cast<const uint16_t*>(bytes.data())[i];
            default: return reinterpret_cast<const uint32_t*>(bytes.data())[i];
        }
    }
};

// Host side of a handle; immutable after encode and shared between clones.
struct HostMatrix {
    bool cser = false;
    int64_t m = 0, n = 0;
    int32_t K = 0;
    int64_t nnz = 0, G = 0;
    int64_t nonempty_groups = 0;
    int64_t max_row_groups = 0;  // largest number of (raw) groups in one row
    std::vector<float> omega;
    std::vector<int64_t> count;
    // len and bits are always set.  A handle encoded on the device leaves `bytes` empty until somebody asks for
    // the arrays on the host (inspection, decode, clone); they are then copied back once from its device copy.
    mutable HostArray colI, omegaPtr, rowPtr, omegaI;
    mutable std::atomic<bool> arrays_on_host{true};
    mutable std::mutex fetch_mutex;
};

// What the kernels see: device pointers into the handle's single allocation.
struct DeviceView {
    const void* colI = nullptr;        // minimal width, followed by 8 KiB of readable zero padding
    const uint32_t* omegaPtr = nullptr; // G + 1
    const uint32_t* rowPtr = nullptr;   // m + 1
    const void* rowInfo = nullptr;      // derived, m + 1 pairs {rowPtr[r], omegaPtr[rowPtr[r]]} as 2 x uint32
    const void* omegaI = nullptr;       // minimal width (CSER)
    const float* omega = nullptr;       // K
    int32_t colI_bits = 16;
    int32_t omegaI_bits = 8;
    int32_t cser = 0;
    int32_t K = 0;
    int64_t m = 0, n = 0;
    int64_t max_row_groups = 0;
    int64_t nnz = 0;
    int64_t nonempty_groups = 0;
    float omega0 = 0.f;
    // the device the arrays live on, as the launchers need it (read once, when the handle is bound to its memory)
    int32_t cus = 256;
    size_t lds_per_block = 64 * 1024;
    // Matrices with rows of unequal length (null / 0 otherwise), for the default batched kernel:
    // row_order[i] = the row served i-th (descending length);
    // split_parts[i] = {row, first position, end position, 0} for every part of a long row but its first;
    // split_rows[j] = {row, its first entry in split_parts, its number of entries, 0}.
    const void* row_order = nullptr;
    const void* split_parts = nullptr;
    const void* split_rows = nullptr;
    uint32_t n_split_parts = 0, n_split_rows = 0;
    uint32_t split_len = 0;  // positions per part
    uint32_t split_min = 0;  // rows with more positions than this are split
    // Strip-major index (derived by cer_prepare_strips; null otherwise): for strip s (strip_rows <= kStripRows consecutive columns of
    // W) and row r, chunks strip_ptr[s * (m + 1) + r] .. strip_ptr[s * (m + 1) + r + 1] of strip_idx; a chunk is eight
    // uint16 entries (rank << 10) | (column - s * strip_rows), the last chunk of a (strip, row) padded with zeros.
    const void* strip_idx = nullptr;
    const uint32_t* strip_ptr = nullptr;
    uint64_t strip_chunks = 0;
    uint32_t strip_rows = 0;
    uint32_t n_strips = 0;
    // Rank table (derived; null unless the codebook has 2 .. 256 values): per row 1 << rank_tab_shift words at a fixed
    // stride, word 0 = the row's first colI position, word k = end of its group of rank k (the previous word when the
    // row has no element of that rank), the same for CER and CSER handles.
    const uint32_t* rank_tab = nullptr;
    int32_t rank_tab_shift = 0;
};
constexpr uint32_t kStripRows = 1024;

// The handle's single device allocation: [colI | 8 KiB readable pad][OmegaPtr u32][rowPtr u32][OmegaI][Omega]
// [row descriptors][rank table], each part 256-byte aligned.  The row descriptors {rowPtr[r], OmegaPtr[rowPtr[r]]} are derived
// from the format arrays: they let a wave find its row's slice of colI with one load instead of two dependent ones.
struct DeviceLayout {
    size_t colI_bytes = 0, omegaI_bytes = 0;
    size_t off_colI = 0, off_optr = 0, off_rptr = 0, off_oi = 0, off_om = 0, off_ri = 0, off_tab = 0, total = 0;
    int32_t tab_shift = 0;  // log2 of the rank table's words per row; 0: no table
    static DeviceLayout make(size_t colI_bytes, int64_t G, int64_t m, size_t omegaI_bytes, int32_t K);
};

// Row order and parts of long rows for the batched product (cer_capi.cpp): whether a matrix of m rows, nnz indexed
// elements and the given longest row gets the table, and its construction from the rows' first colI positions
// (m + 1 entries); a CER_* code.
bool row_schedule_wanted(uint64_t nnz, uint64_t m, uint64_t longest);
int build_row_schedule(cer_matrix* h, const std::vector<uint64_t>& start);

// Host encoder (cer_host.cpp).  Returns a CER_* code.
int encode_host(const float* W, int64_t m, int64_t n, const float* codebook, int32_t K, bool cser,
                std::shared_ptr<HostMatrix>* out);
int decode_host(const HostMatrix& A, float* W_out);
int min_index_bits(uint64_t max_value);

// Per-call choices of cer_matmul_ex (include/cer.h: cer_matmul_opts_t); the defaults are what cer_matmul does.
struct MatmulOptions {
    int path = -1;      // preferred kernel (numbering of cer_matmul_path), -1 = the library's choice
    int tile_cols = 0;  // batched kernels that gather from L2: batch columns per tile, 0 = the library's choice
    uint32_t flags = 0; // CER_OPT_* bits
};
constexpr int kPathStrip = 5;
constexpr uint32_t kOptSumThenMultiply = 1, kOptRowsWhole = 2, kOptXFromGlobal = 4, kOptOneColumnPerLane = 8,
                   kOptShortChunks = 16, kOptLongChunks = 32, kOptNoRankTable = 64;

// HIP launchers (cer_matmul.hip).  Return a hipError_t value as int (0 = success).
// workspace == nullptr: temporaries are stream-ordered allocations.  Otherwise the call allocates nothing: the column
// sums of X (Omega[0] != 0) go to `workspace` (device memory, workspace_floats floats; hipErrorInvalidValue if that
// is fewer than matmul_workspace_floats), and only kernels that need no other temporary are chosen.
int launch_matmul(const DeviceView& v, const float* X, float* Y, int64_t L, void* stream, const MatmulOptions& o,
                  float* workspace = nullptr, size_t workspace_floats = 0);
// The library's fixed workspace on the current device (a __device__ array; nothing is allocated): its device
// address and its size in floats.  A hipError_t value as int.
int static_workspace(float** ptr, size_t* floats);
// Floats of workspace a product of batch L needs (0 when Omega[0] == 0, or when the batch-1 kernel sums X itself).
size_t matmul_workspace_floats(const DeviceView& v, int64_t L, const MatmulOptions& o);
// Which product kernel launch_matmul picks for batch L (numbering of cer_matmul_path).
int matmul_path(const DeviceView& v, int64_t L, const MatmulOptions& o);
// Fills the handle's rank table (if its layout has one) from the format arrays already in device memory; the launch
// is ordered on `stream`.  A hipError_t value as int.
int build_rank_table(const DeviceView& v, void* stream);
int launch_dense(const float* W, const float* X, float* Y, int64_t m, int64_t n, int64_t L, void* stream);
int launch_stream_copy(void* dst, const void* src, int64_t bytes, void* stream);
int launch_stream_read(const void* src, int64_t bytes, void* sink, void* stream);

// Device front-end (frontend.hip): W_dev holds codebook values, or (bits > 0) unquantized weights.
int encode_device(const float* W_dev, int64_t m, int64_t n, const float* codebook, int32_t K, int32_t bits, bool cser,
                  void* stream, float* codebook_out, int32_t* K_out, cer_matrix** out);
int decode_device(const DeviceView& v, float* W_dev, void* stream);
int quantize_device(const float* W_dev, int64_t count, int32_t bits, uint8_t* codes_dev, float* Wq_dev,
                    float* codebook_out, int32_t* K_out, void* stream);

// Remembers a HIP error for cer_last_hip_error() and returns CER_E_HIP (cer_capi.cpp).
int record_hip_error(int hip_error);

// Stream-ordered temporaries (cer_capi.cpp).  They come from a memory pool of the library's own on the current
// device, which keeps what it has handed out once (release threshold: none) -- the default pool gives its memory
// back at every synchronisation, and getting a few hundred megabytes again costs more than the product that needs
// them.  cer_trim() releases what is cached.  Both return a hipError_t value as int.
int temp_alloc(void** p, size_t bytes, void* stream);
int temp_free(void* p, void* stream);

}  // namespace cer

namespace cer {
// Points h's view into `base`, an allocation laid out by `l` that already holds h->host's arrays (cer_capi.cpp).
void bind_device(cer_matrix* h, int dev, void* base, const DeviceLayout& l);
// Makes sure h->host holds the index arrays (copies them back from h's device copy if they are not there yet).
// Thread-safe.  Returns a CER_* code.
int ensure_host_arrays(const cer_matrix* h);
}  // namespace cer

struct cer_matrix {
    std::shared_ptr<const cer::HostMatrix> host;
    int device = -1;          // -1: host-only handle
    void* d_base = nullptr;   // the device allocation of the format arrays
    void* d_split = nullptr;  // row order and parts of long rows (a second, small allocation; null: rows of similar length)
    void* d_strip = nullptr;  // strip-major index (cer_prepare_strips; null: not prepared)
    cer::DeviceLayout layout; // where the arrays sit inside it
    size_t d_bytes = 0;       // its size
    int64_t stream_bytes = 0; // bytes of format arrays a product reads
    cer::DeviceView view;
};

// CSR comparator (csr.hip)
struct csr_host {
    int64_t m = 0, n = 0, nnz = 0;
    std::vector<float> val;
    cer::HostArray colI, rowPtr;
};

struct csr_matrix {
    std::shared_ptr<const csr_host> host;
    int device = -1;
    void* d_base = nullptr;
    const float* d_val = nullptr;
    const void* d_colI = nullptr;
    const uint32_t* d_rowPtr = nullptr;
    int64_t stream_bytes = 0;
};
