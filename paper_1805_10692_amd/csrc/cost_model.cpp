// Host-side analytics: elementary-operation counts, storage and modelled energy of one
// matrix-vector product per format (Sections III-B, IIII and V of the paper).
//
// Counting conventions
//   CER_COUNT_THEOREM  the accounting of Eq. (2), (4), (10), (12) and of the proofs of Theorems 1 and 2 with
//                      c_oth = 0: a row reads one rowPtr entry and one OmegaPtr entry per group (the previous
//                      end is carried), one addition per element that takes part (dense: every element,
//                      CSR / CER / CSER: every indexed element), one multiplication and one Omega read per
//                      non-empty group.
//   CER_COUNT_EXAMPLE  the hand count of Section III-B for a single row: both ends of the row's pointer
//                      range are read (2 rowPtr entries, groups + 1 OmegaPtr entries) and summing k
//                      terms costs k - 1 additions.  (Dense 48, CSR 32, CER 24 for the example row.)
// Energy: every count is priced with Table I (45 nm CMOS, pJ): 32-bit float add 0.9, mul 3.7; a read or
// write costs by the width of the value and the size of the array that holds it (< 8 KB, < 32 KB, < 1 MB,
// larger).  The 16-bit cell of the last row is printed as 5000.0 in the paper; the caption's linear
// interpolation gives 500.0, which is used here.
#include <cstdint>

#include "../../include/cer.h"
#include "cer_internal.hpp"

namespace {

double rw_cost(int bits, double array_bytes) {
    static const double table[4][3] = {{1.25, 2.5, 5.0}, {2.5, 5.0, 10.0}, {12.5, 25.0, 50.0}, {250.0, 500.0, 1000.0}};
    const int col = bits <= 8 ? 0 : (bits <= 16 ? 1 : 2);
    const int row = array_bytes < 8.0 * 1024 ? 0 : (array_bytes < 32.0 * 1024 ? 1 : (array_bytes < 1024.0 * 1024 ? 2 : 3));
    return table[row][col];
}
constexpr double kAdd32 = 0.9, kMul32 = 3.7;

void price(cer_cost_t* c, int64_t m, int64_t n, double weight_bytes, int omega_bits, double omega_bytes, int coli_bits,
           double coli_bytes, int optr_bits, double optr_bytes, int rptr_bits, double rptr_bytes, int oi_bits,
           double oi_bytes) {
    c->energy_pj = (double)c->read_weight * rw_cost(32, weight_bytes) + (double)c->read_omega * rw_cost(omega_bits, omega_bytes) +
                   (double)c->read_colI * rw_cost(coli_bits, coli_bytes) + (double)c->read_omegaPtr * rw_cost(optr_bits, optr_bytes) +
                   (double)c->read_rowPtr * rw_cost(rptr_bits, rptr_bytes) + (double)c->read_omegaI * rw_cost(oi_bits, oi_bytes) +
                   (double)c->read_input * rw_cost(32, 4.0 * (double)n) + (double)c->write * rw_cost(32, 4.0 * (double)m) +
                   (double)c->mul * kMul32 + (double)c->add * kAdd32;
}

}  // namespace

extern "C" {

int dense_cost_model(int64_t m, int64_t n, int convention, cer_cost_t* c) {
    if (!c || m < 0 || n < 0 || (convention != CER_COUNT_THEOREM && convention != CER_COUNT_EXAMPLE)) return CER_E_INVALID;
    *c = cer_cost_t{};
    const int64_t N = m * n;
    c->read_weight = N;
    c->read_input = N;
    c->mul = N;
    c->add = convention == CER_COUNT_THEOREM ? N : (n > 0 ? m * (n - 1) : 0);
    c->write = m;
    c->storage_bits = N * 32;
    price(c, m, n, 4.0 * (double)N, 32, 0, 8, 0, 8, 0, 8, 0, 8, 0);
    return CER_OK;
}

int csr_cost_model(const csr_handle_t* h, int convention, cer_cost_t* c) {
    if (!h || !c || (convention != CER_COUNT_THEOREM && convention != CER_COUNT_EXAMPLE)) return CER_E_INVALID;
    const csr_host& A = *h->host;
    *c = cer_cost_t{};
    c->read_weight = A.nnz;
    c->read_colI = A.nnz;
    c->read_input = A.nnz;
    c->mul = A.nnz;
    c->write = A.m;
    if (convention == CER_COUNT_THEOREM) {
        c->read_rowPtr = A.m;
        c->add = A.nnz;
    } else {
        c->read_rowPtr = 2 * A.m;
        for (int64_t r = 0; r < A.m; ++r) {
            const int64_t k = (int64_t)A.rowPtr.at(r + 1) - (int64_t)A.rowPtr.at(r);
            if (k > 0) c->add += k - 1;
        }
    }
    c->storage_bits = A.nnz * 32 + A.colI.len * A.colI.bits + A.rowPtr.len * A.rowPtr.bits;
    price(c, A.m, A.n, 4.0 * (double)A.nnz, 32, 0, A.colI.bits, (double)A.colI.bytes.size(), 8, 0, A.rowPtr.bits,
          (double)A.rowPtr.bytes.size(), 8, 0);
    return CER_OK;
}

int cer_cost_model(const cer_handle_t* h, int convention, cer_cost_t* c) {
    if (!h || !c || (convention != CER_COUNT_THEOREM && convention != CER_COUNT_EXAMPLE)) return CER_E_INVALID;
    try {
        const int rc = cer::ensure_host_arrays(h);
        if (rc != CER_OK) return rc;
    } catch (...) {
        return CER_E_NOMEM;
    }
    const cer::HostMatrix& A = *h->host;
    *c = cer_cost_t{};
    c->read_colI = A.nnz;
    c->read_input = A.nnz;
    c->read_omega = A.nonempty_groups;  // one value per non-empty group
    c->mul = A.nonempty_groups;
    c->write = A.m;
    if (A.cser) c->read_omegaI = A.G;
    if (convention == CER_COUNT_THEOREM) {
        c->read_rowPtr = A.m;
        c->read_omegaPtr = A.G;
        c->add = A.nnz;
    } else {
        c->read_rowPtr = 2 * A.m;
        c->read_omegaPtr = A.G + A.m;
        for (int64_t r = 0; r < A.m; ++r) {
            const int64_t g0 = (int64_t)A.rowPtr.at(r), g1 = (int64_t)A.rowPtr.at(r + 1);
            const int64_t k = (int64_t)A.omegaPtr.at(g1) - (int64_t)A.omegaPtr.at(g0);
            if (k > 0) c->add += k - 1;  // k gathered inputs in this row: k - groups adds inside, groups - 1 across
        }
    }
    c->storage_bits = cer_storage_bits(h);
    // a non-zero most frequent value adds n additions and one multiplication to the whole product (Appendix A-A1)
    if (A.K > 0 && A.omega[0] != 0.0f && A.m > 0) {
        c->read_input += A.n;
        c->add += A.n + A.m;
        c->mul += 1;
        c->read_omega += 1;
    }
    price(c, A.m, A.n, 0, 32, 4.0 * (double)A.K, A.colI.bits, (double)A.colI.bytes.size(), A.omegaPtr.bits,
          (double)A.omegaPtr.bytes.size(), A.rowPtr.bits, (double)A.rowPtr.bytes.size(), A.omegaI.bits,
          (double)A.omegaI.bytes.size());
    return CER_OK;
}

}  // extern "C"
