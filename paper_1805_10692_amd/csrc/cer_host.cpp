// Host-side encoder and decoder of the CER / CSER formats (Section III-A of the paper).
//
// The encoder is a three-pass, row-parallel counting sort:
//   pass 1  element -> codebook symbol through a hash of the fp32 bit pattern; global histogram
//   (order) symbols ranked by count (Section III-A step 1: frequency-major Omega)
//   pass 2  per row: histogram over ranks -> number of indexed elements and of groups
//   (scan)  exclusive prefix sums give every row its slice of colI / OmegaPtr / OmegaI
//   pass 3  per row: scatter the columns into their rank bucket (ascending inside a bucket because
//           columns are visited in order) and write the bucket boundaries as the row's pointers
// Conversion cost is O(m.n), as the paper notes in Section V.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>

#include "../../include/cer.h"
#include "cer_internal.hpp"

namespace cer {
namespace {

inline uint32_t value_bits(float v) {
    if (v == 0.0f) v = 0.0f;  // -0.0 and +0.0 are one value, stored as +0.0
    uint32_t u;
    std::memcpy(&u, &v, 4);
    return u;
}

// Open-addressing table: fp32 bit pattern -> position in the caller's codebook.
class SymbolTable {
public:
    explicit SymbolTable(int32_t K) {
        size_t cap = 16;
        while (cap < (size_t)K * 4) cap <<= 1;
        mask_ = cap - 1;
        keys_.assign(cap, 0);
        vals_.assign(cap, -1);
    }
    // false if the key is already present
    bool insert(uint32_t key, int32_t val) {
        size_t h = slot(key);
        while (vals_[h] >= 0) {
            if (keys_[h] == key) return false;
            h = (h + 1) & mask_;
        }
        keys_[h] = key;
        vals_[h] = val;
        return true;
    }
    int32_t find(uint32_t key) const {
        size_t h = slot(key);
        while (vals_[h] >= 0) {
            if (keys_[h] == key) return vals_[h];
            h = (h + 1) & mask_;
        }
        return -1;
    }

private:
    size_t slot(uint32_t key) const { return (size_t)((key * 0x9E3779B1u) >> 7) & mask_; }
    size_t mask_;
    std::vector<uint32_t> keys_;
    std::vector<int32_t> vals_;
};

int worker_count(int64_t rows) {
    unsigned hw = std::thread::hardware_concurrency();
    int t = (int)std::min<unsigned>(hw ? hw : 1, 16);
    return (int)std::max<int64_t>(1, std::min<int64_t>(t, rows));
}

template <typename F>
void parallel_rows(int64_t m, int nthreads, F&& body) {
    if (nthreads <= 1 || m < 2) {
        body(0, (int64_t)0, m);
        return;
    }
    std::vector<std::thread> pool;
    int64_t per = (m + nthreads - 1) / nthreads;
    for (int t = 0; t < nthreads; ++t) {
        int64_t r0 = std::min<int64_t>(m, t * per), r1 = std::min<int64_t>(m, r0 + per);
        pool.emplace_back([&body, t, r0, r1] { body(t, r0, r1); });
    }
    for (auto& th : pool) th.join();
}

void narrow(const std::vector<uint32_t>& src, int bits, HostArray* dst) {
    dst->len = (int64_t)src.size();
    dst->bits = bits;
    dst->bytes.resize(src.size() * (size_t)(bits / 8));
    if (bits == 8) {
        for (size_t i = 0; i < src.size(); ++i) dst->bytes[i] = (uint8_t)src[i];
    } else if (bits == 16) {
        auto* p = reinterpret_cast<uint16_t*>(dst->bytes.data());
        for (size_t i = 0; i < src.size(); ++i) p[i] = (uint16_t)src[i];
    } else {
        std::memcpy(dst->bytes.data(), src.data(), src.size() * 4);
    }
}

}  // namespace

int min_index_bits(uint64_t max_value) {
    return max_value <= 0xFFu ? 8 : (max_value <= 0xFFFFu ? 16 : 32);
}

int encode_host(const float* W, int64_t m, int64_t n, const float* codebook, int32_t Kc, bool cser,
                std::shared_ptr<HostMatrix>* out) {
    if (n > (int64_t)0xFFFFFFFFll) return CER_E_TOO_LARGE;
    const int64_t N = m * n;

    SymbolTable table(Kc);
    for (int32_t k = 0; k < Kc; ++k) {
        if (!std::isfinite(codebook[k])) return CER_E_BAD_CODEBOOK;
        if (!table.insert(value_bits(codebook[k]), k)) return CER_E_BAD_CODEBOOK;
    }

    // pass 1: symbols and the global histogram
    std::vector<uint32_t> sym((size_t)N);
    const int T = worker_count(m);
    std::vector<std::vector<int64_t>> hist((size_t)T, std::vector<int64_t>((size_t)Kc, 0));
    std::atomic<bool> missing{false};
    parallel_rows(m, T, [&](int t, int64_t r0, int64_t r1) {
        auto& h = hist[(size_t)t];
        uint32_t last_key = 0;
        int32_t last_sym = -1;
        for (int64_t i = r0 * n; i < r1 * n; ++i) {
            uint32_t key = value_bits(W[i]);
            if (last_sym < 0 || key != last_key) {
                int32_t s = table.find(key);
                if (s < 0) { missing.store(true); return; }
                last_key = key;
                last_sym = s;
            }
            sym[(size_t)i] = (uint32_t)last_sym;
            ++h[(size_t)last_sym];
        }
    });
    if (missing.load()) return CER_E_NOT_IN_CODEBOOK;
    std::vector<int64_t> total((size_t)Kc, 0);
    for (auto& h : hist)
        for (int32_t k = 0; k < Kc; ++k) total[(size_t)k] += h[(size_t)k];

    // Omega: occurring symbols by count, highest first; stable, so equal counts keep codebook order
    std::vector<int32_t> order;
    for (int32_t k = 0; k < Kc; ++k)
        if (total[(size_t)k] > 0) order.push_back(k);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return total[(size_t)a] > total[(size_t)b]; });
    const int32_t K = (int32_t)order.size();
    std::vector<uint32_t> rank_of((size_t)std::max(Kc, 1), 0);
    auto A = std::make_shared<HostMatrix>();
    A->cser = cser; A->m = m; A->n = n; A->K = K;
    A->omega.resize((size_t)K);
    A->count.resize((size_t)K);
    for (int32_t k = 0; k < K; ++k) {
        rank_of[(size_t)order[(size_t)k]] = (uint32_t)k;
        float v = codebook[order[(size_t)k]];
        A->omega[(size_t)k] = (v == 0.0f) ? 0.0f : v;
        A->count[(size_t)k] = total[(size_t)order[(size_t)k]];
    }
    for (auto& s : sym) s = rank_of[s];  // from here on: rank of every element

    // pass 2: per-row sizes
    std::vector<uint64_t> row_nnz((size_t)m + 1, 0), row_groups((size_t)m + 1, 0);
    std::vector<int64_t> nonempty_part((size_t)T, 0);
    parallel_rows(m, T, [&](int t, int64_t r0, int64_t r1) {
        std::vector<uint32_t> c((size_t)std::max(K, 1));
        for (int64_t r = r0; r < r1; ++r) {
            std::fill(c.begin(), c.end(), 0u);
            const uint32_t* s = sym.data() + r * n;
            for (int64_t j = 0; j < n; ++j) ++c[s[j]];
            uint64_t present = 0, top = 0;
            for (int32_t k = 1; k < K; ++k)
                if (c[(size_t)k]) { ++present; top = (uint64_t)k; }
            row_nnz[(size_t)r] = (uint64_t)n - c[0];
            row_groups[(size_t)r] = cser ? present : top;
            nonempty_part[(size_t)t] += (int64_t)present;
        }
    });
    // exclusive scans
    uint64_t acc_n = 0, acc_g = 0;
    for (int64_t r = 0; r <= m; ++r) {
        uint64_t a = row_nnz[(size_t)r], g = row_groups[(size_t)r];
        row_nnz[(size_t)r] = acc_n;
        row_groups[(size_t)r] = acc_g;
        acc_n += a;
        acc_g += g;
    }
    // the kernels address colI and OmegaPtr with 32-bit offsets and read ahead of a row's end
    const uint64_t limit = 0xFFFFFFFFull - 65536;
    if (acc_n > limit || acc_g > limit) return CER_E_TOO_LARGE;
    A->nnz = (int64_t)acc_n;
    A->G = (int64_t)acc_g;
    A->nonempty_groups = std::accumulate(nonempty_part.begin(), nonempty_part.end(), (int64_t)0);
    for (int64_t r = 0; r < m; ++r)
        A->max_row_groups = std::max<int64_t>(A->max_row_groups, (int64_t)(row_groups[(size_t)r + 1] - row_groups[(size_t)r]));

    // pass 3: fill
    std::vector<uint32_t> colI((size_t)acc_n), omegaPtr((size_t)acc_g + 1), rowPtr((size_t)m + 1),
        omegaI(cser ? (size_t)acc_g : 0);
    omegaPtr[0] = 0;
    for (int64_t r = 0; r <= m; ++r) rowPtr[(size_t)r] = (uint32_t)row_groups[(size_t)r];
    parallel_rows(m, T, [&](int, int64_t r0, int64_t r1) {
        std::vector<uint32_t> start((size_t)std::max(K, 1) + 1), fill((size_t)std::max(K, 1));
        for (int64_t r = r0; r < r1; ++r) {
            const uint32_t* s = sym.data() + r * n;
            std::fill(start.begin(), start.end(), 0u);
            for (int64_t j = 0; j < n; ++j) ++start[(size_t)s[j] + 1];
            start[1] = 0;  // rank 0 owns no indices
            for (int32_t k = 2; k <= K; ++k) start[(size_t)k] += start[(size_t)k - 1];
            // start[k] = offset of rank k's bucket inside the row, start[K] = row nnz (K >= 1)
            const uint32_t base = (uint32_t)row_nnz[(size_t)r];
            for (int32_t k = 1; k < K; ++k) fill[(size_t)k] = start[(size_t)k];
            for (int64_t j = 0; j < n; ++j) {
                uint32_t k = s[j];
                if (k) colI[(size_t)base + fill[k]++] = (uint32_t)j;
            }
            uint64_t g = row_groups[(size_t)r];
            const uint64_t g_end = row_groups[(size_t)r + 1];
            for (int32_t k = 1; k < K && g < g_end; ++k) {
                uint32_t b0 = start[(size_t)k], b1 = (k + 1 <= K) ? start[(size_t)k + 1] : b0;
                if (cser) {
                    if (b1 == b0) continue;
                    omegaI[(size_t)g] = (uint32_t)k;
                }
                omegaPtr[(size_t)++g] = base + b1;
            }
        }
    });

    narrow(colI, min_index_bits(n > 0 ? (uint64_t)(n - 1) : 0), &A->colI);
    narrow(omegaPtr, min_index_bits((uint64_t)A->nnz), &A->omegaPtr);
    narrow(rowPtr, min_index_bits((uint64_t)A->G), &A->rowPtr);
    if (cser) narrow(omegaI, min_index_bits(K > 0 ? (uint64_t)(K - 1) : 0), &A->omegaI);
    *out = std::move(A);
    return CER_OK;
}

int decode_host(const HostMatrix& A, float* W) {
    const int64_t N = A.m * A.n;
    if (N == 0) return CER_OK;
    if (A.K < 1) return CER_E_INVALID;
    std::fill(W, W + N, A.omega[0]);
    parallel_rows(A.m, worker_count(A.m), [&](int, int64_t r0, int64_t r1) {
        for (int64_t r = r0; r < r1; ++r) {
            float* row = W + r * A.n;
            const int64_t g0 = (int64_t)A.rowPtr.at(r), g1 = (int64_t)A.rowPtr.at(r + 1);
            for (int64_t g = g0; g < g1; ++g) {
                const int64_t rank = A.cser ? (int64_t)A.omegaI.at(g) : g - g0 + 1;
                const float v = A.omega[(size_t)rank];
                const int64_t e = (int64_t)A.omegaPtr.at(g + 1);
                for (int64_t i = (int64_t)A.omegaPtr.at(g); i < e; ++i) row[A.colI.at(i)] = v;
            }
        }
    });
    return CER_OK;
}

}  // namespace cer
