// CPU oracle for the DCT hard-thresholding path.  TEST INFRASTRUCTURE ONLY:
// it is slow on purpose, single-threaded, and is used by the tests, by the
// smoke check and by the benchmark's cpu_baseline leg.  It shares no code with
// the HIP library and the product never calls it.
//
// What it computes is the plain definition in the paper:
//   * DCT-DP (Algorithm 1: the sort of the magnitudes, the pick of tau at rank
//     floor(N*eta), the mask of the magnitudes >= tau, the masked gradient): the threshold is an order
//     statistic of the magnitudes found by a FULL SORT of a copy (the
//     copy-and-sort routine of Sec. 3.3), the mask is a scalar filter.
//   * DCT-MP (Algorithm 2, forward loop over rows and the masked gradient of the backward pass):
//     per row, the k largest magnitudes by a partial sort; the backward pass
//     reuses the forward mask (Sec. 2.2).
//
//   * Error feedback (Algorithm 1: the residual is added to the gradient before the
//     selection and becomes what the mask removed after it; Fig. 3): the
//     *_ef functions add the residual first, select / filter the sum, and return
//     the new residual.
//
//   * Receiver side (Sec. 2.1 names decompression next to compression as the overhead; Algorithm 2: the
//     next worker consumes the masked activations): oracle_scatter / oracle_rowscatter put the
//     pairs back into a dense tensor, by assignment into zeros or (fp32) by addition.
//
// Readings fixed where the paper is silent (listed in the design notes too):
//   * the caller passes the integer number kept, k; no fraction is rounded here;
//   * magnitude order is the order of key(x) = bit pattern of x with the sign bit
//     cleared, read as unsigned (equal to the order of |x| for non-NaN x;
//     -0 == +0; denormals are not flushed; NaNs rank above infinity);
//   * position i precedes position j when key[i] > key[j], or the keys are equal
//     and i < j (ties go to the lower index);
//   * mode GE keeps every key >= tau (the paper's mask, count may exceed k);
//     mode EXACT keeps key > tau plus the first tie_quota ties in index order
//     (exactly k survivors on the vector tau was selected from);
//   * survivors are emitted as (int32 index, value) in ascending index order,
//     values copied bit for bit;
//   * error feedback is defined for fp32: w[i] = g[i] + e[i] is one IEEE-754
//     binary32 addition, round to nearest even, denormals kept.  The new residual
//     is the part of w that was not delivered: +0 where (i, w[i]) was written to
//     the output, w[i] (bit for bit) everywhere else -- this includes entries that
//     pass the mask but do not fit into `capacity`, which therefore are not lost.
//
// Parity status: every function below is pinned by tests that do not call it to
// produce their expected values (O(N^2) rank counting on tiny inputs, closed
// forms, hand-worked fixtures, numpy/torch library routines on tie-free data).
// The paper prints no worked numeric example, so no pin comes from its text.

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <utility>
#include <vector>

namespace {

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_GE_TAU = 0, ORACLE_EXACT_K = 1 };

inline uint32_t key_at(const void* base, int dtype, uint64_t i) {
    if (dtype == ORACLE_F32) {
        uint32_t bits;
        std::memcpy(&bits, static_cast<const unsigned char*>(base) + 4 * i, 4);
        return bits & 0x7FFFFFFFu;
    }
    uint16_t bits;
    std::memcpy(&bits, static_cast<const unsigned char*>(base) + 2 * i, 2);
    return static_cast<uint32_t>(bits & 0x7FFFu);
}

inline size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

struct KeyPos {
    uint32_t key;
    uint32_t pos;
};

// The total order of the paper's sort with ties resolved to the lower index.
inline bool precedes(const KeyPos& a, const KeyPos& b) {
    if (a.key != b.key) return a.key > b.key;
    return a.pos < b.pos;
}

}  // namespace

extern "C" {

// Algorithm 1, threshold selection: copy, full sort, read the k-th entry.
// out = {tau_key, n_gt, n_eq, tie_quota}.  Returns 0, or 1 on invalid arguments.
int oracle_select_threshold(const void* g, int dtype, uint64_t n, uint64_t k, uint32_t* out) {
    if (!g || !out || n == 0 || k == 0 || k > n || n > 0x7FFFFFFFull) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    std::vector<KeyPos> a(n);
    for (uint64_t i = 0; i < n; ++i) {
        a[i].key = key_at(g, dtype, i);
        a[i].pos = static_cast<uint32_t>(i);
    }
    std::sort(a.begin(), a.end(), precedes);
    const uint32_t tau = a[k - 1].key;
    uint64_t n_gt = 0, n_eq = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t key = key_at(g, dtype, i);
        if (key > tau) ++n_gt;
        if (key == tau) ++n_eq;
    }
    out[0] = tau;
    out[1] = static_cast<uint32_t>(n_gt);
    out[2] = static_cast<uint32_t>(n_eq);
    out[3] = static_cast<uint32_t>(k - n_gt);
    return 0;
}

// Same order statistic through std::nth_element (no full sort): timed by the
// benchmark as a stronger single-thread CPU baseline; tests check it equals the
// full-sort result.
int oracle_select_threshold_nth(const void* g, int dtype, uint64_t n, uint64_t k, uint32_t* out) {
    if (!g || !out || n == 0 || k == 0 || k > n || n > 0x7FFFFFFFull) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    std::vector<uint32_t> a(n);
    for (uint64_t i = 0; i < n; ++i) a[i] = key_at(g, dtype, i);
    std::nth_element(a.begin(), a.begin() + (k - 1), a.end(), [](uint32_t x, uint32_t y) { return x > y; });
    const uint32_t tau = a[k - 1];
    uint64_t n_gt = 0, n_eq = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t key = key_at(g, dtype, i);
        if (key > tau) ++n_gt;
        if (key == tau) ++n_eq;
    }
    out[0] = tau;
    out[1] = static_cast<uint32_t>(n_gt);
    out[2] = static_cast<uint32_t>(n_eq);
    out[3] = static_cast<uint32_t>(k - n_gt);
    return 0;
}

// Algorithm 1, mask and compressed gradient: scalar filter in index order.
// thr = {tau_key, n_gt, n_eq, tie_quota}.  Writes at most `capacity` pairs (the
// first ones in index order) and the full survivor count to *count.
int oracle_threshold_compact(const void* g, int dtype, uint64_t n, const uint32_t* thr, int mode,
                             int32_t* idx_out, void* val_out, uint64_t capacity, uint64_t* count) {
    if (!g || !thr || !count || n == 0 || n > 0x7FFFFFFFull) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    if (mode != ORACLE_GE_TAU && mode != ORACLE_EXACT_K) return 1;
    if (capacity > 0 && (!idx_out || !val_out)) return 1;
    const uint32_t tau = thr[0];
    const uint32_t quota = thr[3];
    const size_t es = elem_size(dtype);
    uint64_t kept = 0;
    uint32_t ties_kept = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t key = key_at(g, dtype, i);
        bool keep;
        if (mode == ORACLE_GE_TAU) {
            keep = key >= tau;
        } else if (key > tau) {
            keep = true;
        } else if (key == tau && ties_kept < quota) {
            keep = true;
            ++ties_kept;
        } else {
            keep = false;
        }
        if (!keep) continue;
        if (kept < capacity) {
            idx_out[kept] = static_cast<int32_t>(i);
            std::memcpy(static_cast<unsigned char*>(val_out) + es * kept,
                        static_cast<const unsigned char*>(g) + es * i, es);
        }
        ++kept;
    }
    *count = kept;
    return 0;
}

// Algorithm 2, forward pass: for each row, the k entries that come first in the
// magnitude order (partial sort), re-ordered by column; values copied; tau_out
// (optional) receives the magnitude of the k-th one in the row's dtype.
int oracle_rowtopk_fwd(const void* x, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                       int32_t* idx_out, void* val_out, void* tau_out) {
    if (!x || !idx_out || !val_out || B == 0 || D == 0 || k == 0 || k > D || row_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    std::vector<KeyPos> a(D);
    std::vector<uint32_t> cols(k);
    for (uint32_t b = 0; b < B; ++b) {
        const unsigned char* row = static_cast<const unsigned char*>(x) + es * row_stride * b;
        for (uint32_t c = 0; c < D; ++c) {
            a[c].key = key_at(row, dtype, c);
            a[c].pos = c;
        }
        std::partial_sort(a.begin(), a.begin() + k, a.end(), precedes);
        for (uint32_t j = 0; j < k; ++j) cols[j] = a[j].pos;
        const uint32_t tau = a[k - 1].key;
        std::sort(cols.begin(), cols.end());
        for (uint32_t j = 0; j < k; ++j) {
            const uint64_t o = static_cast<uint64_t>(b) * k + j;
            idx_out[o] = static_cast<int32_t>(cols[j]);
            std::memcpy(static_cast<unsigned char*>(val_out) + es * o, row + es * cols[j], es);
        }
        if (tau_out) {
            if (dtype == ORACLE_F32) {
                std::memcpy(static_cast<unsigned char*>(tau_out) + 4ull * b, &tau, 4);
            } else {
                const uint16_t t16 = static_cast<uint16_t>(tau);
                std::memcpy(static_cast<unsigned char*>(tau_out) + 2ull * b, &t16, 2);
            }
        }
    }
    return 0;
}

// Algorithm 2, backward pass: X_grad through the forward mask, i.e. a gather
// of dy at the forward indices.  No new selection takes place.
int oracle_rowtopk_bwd(const void* dy, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                       const int32_t* idx, void* dval_out) {
    if (!dy || !idx || !dval_out || B == 0 || D == 0 || k == 0 || k > D || row_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    for (uint32_t b = 0; b < B; ++b) {
        const unsigned char* row = static_cast<const unsigned char*>(dy) + es * row_stride * b;
        for (uint32_t j = 0; j < k; ++j) {
            const uint64_t o = static_cast<uint64_t>(b) * k + j;
            const int32_t c = idx[o];
            if (c < 0 || static_cast<uint32_t>(c) >= D) return 2;
            std::memcpy(static_cast<unsigned char*>(dval_out) + es * o, row + es * static_cast<uint32_t>(c), es);
        }
    }
    return 0;
}

// ---- Algorithm 1 with error feedback (fp32) --------------------------------

// The corrected gradient (Algorithm 1, first step with error feedback): one binary32 addition per element.  The sum is
// formed in binary64, where it is exact or correctly rounded with far more than
// 2*24+2 digits, and rounded once to binary32: the same value as a single
// round-to-nearest-even binary32 addition.
int oracle_ef_accumulate(const float* g, const float* e, uint64_t n, float* w) {
    if (!g || !e || !w || n == 0 || n > 0x7FFFFFFFull) return 1;
    for (uint64_t i = 0; i < n; ++i) {
        const double wide = static_cast<double>(g[i]) + static_cast<double>(e[i]);
        w[i] = static_cast<float>(wide);
    }
    return 0;
}

// Threshold selection on the corrected gradient: tau = k-th largest |g + e|.
int oracle_ef_select_threshold(const float* g, const float* e, uint64_t n, uint64_t k, uint32_t* out) {
    if (!g || !e || !out || n == 0 || n > 0x7FFFFFFFull) return 1;
    std::vector<float> w(n);
    if (oracle_ef_accumulate(g, e, n, w.data()) != 0) return 1;
    return oracle_select_threshold(w.data(), ORACLE_F32, n, k, out);
}

// Mask, compressed gradient and new residual (Algorithm 1, the residual update after the mask):
// filter w = g + e in index order exactly as oracle_threshold_compact filters g;
// e_out[i] = +0 where the pair (i, w[i]) was written, w[i] otherwise.
int oracle_ef_threshold_compact(const float* g, const float* e_in, uint64_t n, const uint32_t* thr, int mode,
                                int32_t* idx_out, float* val_out, uint64_t capacity, uint64_t* count,
                                float* e_out) {
    if (!g || !e_in || !e_out || !thr || !count || n == 0 || n > 0x7FFFFFFFull) return 1;
    if (mode != ORACLE_GE_TAU && mode != ORACLE_EXACT_K) return 1;
    if (capacity > 0 && (!idx_out || !val_out)) return 1;
    std::vector<float> w(n);
    if (oracle_ef_accumulate(g, e_in, n, w.data()) != 0) return 1;
    const uint32_t tau = thr[0];
    const uint32_t quota = thr[3];
    uint64_t kept = 0;
    uint32_t ties_kept = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t key = key_at(w.data(), ORACLE_F32, i);
        bool keep;
        if (mode == ORACLE_GE_TAU) {
            keep = key >= tau;
        } else if (key > tau) {
            keep = true;
        } else if (key == tau && ties_kept < quota) {
            keep = true;
            ++ties_kept;
        } else {
            keep = false;
        }
        bool written = false;
        if (keep) {
            if (kept < capacity) {
                idx_out[kept] = static_cast<int32_t>(i);
                val_out[kept] = w[i];
                written = true;
            }
            ++kept;
        }
        e_out[i] = written ? 0.0f : w[i];
    }
    *count = kept;
    return 0;
}

// ---- receiver side: decompression -------------------------------------------
// What the next worker / the parameter server does with a compressed message
// (Sec. 2.1 counts compressing and decompressing as the overhead of DCT; in
// Algorithm 2 the next worker consumes the masked activations): put the pairs back into a
// dense tensor.  mode 0 (assign): out = 0, then out[idx[j]] = val[j];
// mode 1 (add, fp32 only): out[idx[j]] = out[idx[j]] + val[j], one binary32
// addition each (the server-side sum of the workers' sparse gradients).
// Pairs are applied in order j = 0 .. count-1; an index outside [0, n) is skipped.
int oracle_scatter(const int32_t* idx, const void* val, uint64_t count, int dtype, uint64_t n, void* out,
                   int mode) {
    if (!out || n == 0 || (count > 0 && (!idx || !val))) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    if (mode != 0 && !(mode == 1 && dtype == ORACLE_F32)) return 1;
    const size_t es = elem_size(dtype);
    if (mode == 0) std::memset(out, 0, es * n);
    for (uint64_t j = 0; j < count; ++j) {
        const int32_t i = idx[j];
        if (i < 0 || static_cast<uint64_t>(i) >= n) continue;
        unsigned char* dst = static_cast<unsigned char*>(out) + es * static_cast<uint64_t>(i);
        const unsigned char* src = static_cast<const unsigned char*>(val) + es * j;
        if (mode == 0) {
            std::memcpy(dst, src, es);
        } else {
            float a, b;
            std::memcpy(&a, dst, 4);
            std::memcpy(&b, src, 4);
            const float sum = static_cast<float>(static_cast<double>(a) + static_cast<double>(b));
            std::memcpy(dst, &sum, 4);
        }
    }
    return 0;
}

// Dense [B, D] matrix (row stride out_stride elements) from the per-row lists
// of Algorithm 2: zero everywhere, out[b, idx[b, j]] = val[b, j].  Elements
// between D and out_stride are not touched.  A column outside [0, D) is skipped.
int oracle_rowscatter(const int32_t* idx, const void* val, int dtype, uint32_t B, uint32_t D, uint32_t k,
                      void* out, uint64_t out_stride) {
    if (!idx || !val || !out || B == 0 || D == 0 || k == 0 || out_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    for (uint32_t b = 0; b < B; ++b) {
        unsigned char* row = static_cast<unsigned char*>(out) + es * out_stride * b;
        std::memset(row, 0, es * D);
        for (uint32_t j = 0; j < k; ++j) {
            const uint64_t o = static_cast<uint64_t>(b) * k + j;
            const int32_t c = idx[o];
            if (c < 0 || static_cast<uint32_t>(c) >= D) continue;
            std::memcpy(row + es * static_cast<uint32_t>(c), static_cast<const unsigned char*>(val) + es * o, es);
        }
    }
    return 0;
}

// ---- Algorithm 2 with the mask sent as a bitmap -------------------------------
// Algorithm 2 sends the masked activations and the mask M.  Here M travels literally as a
// bitmap: ceil(D/32) 32-bit words per row, bit (c mod 32) of word (c div 32) set
// iff column c is kept, plus the k kept values in ascending column order.  The
// kept set is the one oracle_rowtopk_fwd computes; only the encoding differs.
int oracle_rowtopk_fwd_bitmask(const void* x, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                               uint32_t* mask_out, void* val_out, void* tau_out) {
    if (!mask_out) return 1;
    std::vector<int32_t> idx(static_cast<size_t>(B) * k);
    const int rc = oracle_rowtopk_fwd(x, dtype, B, D, row_stride, k, idx.data(), val_out, tau_out);
    if (rc != 0) return rc;
    const uint32_t words = (D + 31) / 32;
    for (uint32_t b = 0; b < B; ++b) {
        uint32_t* m = mask_out + static_cast<size_t>(b) * words;
        for (uint32_t w = 0; w < words; ++w) m[w] = 0;
        for (uint32_t j = 0; j < k; ++j) {
            const uint32_t c = static_cast<uint32_t>(idx[static_cast<size_t>(b) * k + j]);
            m[c / 32] |= 1u << (c % 32);
        }
    }
    return 0;
}

// Backward through a bitmap mask: dval[b, j] = dy[b, column of the j-th set bit
// of row b's mask] for j < min(k, set bits); the rest of the row's k slots are 0.
int oracle_rowtopk_bwd_bitmask(const void* dy, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                               const uint32_t* mask, void* dval_out) {
    if (!dy || !mask || !dval_out || B == 0 || D == 0 || k == 0 || k > D || row_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    const uint32_t words = (D + 31) / 32;
    for (uint32_t b = 0; b < B; ++b) {
        const unsigned char* row = static_cast<const unsigned char*>(dy) + es * row_stride * b;
        unsigned char* out = static_cast<unsigned char*>(dval_out) + es * static_cast<size_t>(b) * k;
        std::memset(out, 0, es * k);
        uint32_t j = 0;
        for (uint32_t c = 0; c < D && j < k; ++c) {
            if ((mask[static_cast<size_t>(b) * words + c / 32] >> (c % 32)) & 1u) {
                std::memcpy(out + es * j, row + es * c, es);
                ++j;
            }
        }
    }
    return 0;
}

// Receiver side for the bitmap encoding: dense row = zeros with the j-th value
// at the column of the j-th set bit (j < k).
int oracle_rowscatter_bitmask(const uint32_t* mask, const void* val, int dtype, uint32_t B, uint32_t D, uint32_t k,
                              void* out, uint64_t out_stride) {
    if (!mask || !val || !out || B == 0 || D == 0 || k == 0 || out_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    const uint32_t words = (D + 31) / 32;
    for (uint32_t b = 0; b < B; ++b) {
        unsigned char* row = static_cast<unsigned char*>(out) + es * out_stride * b;
        std::memset(row, 0, es * D);
        uint32_t j = 0;
        for (uint32_t c = 0; c < D && j < k; ++c) {
            if ((mask[static_cast<size_t>(b) * words + c / 32] >> (c % 32)) & 1u) {
                std::memcpy(row + es * c, static_cast<const unsigned char*>(val) + es * (static_cast<size_t>(b) * k + j), es);
                ++j;
            }
        }
    }
    return 0;
}

// ---- Algorithm 2 with the mask sent as 16-bit column indices -------------------
// The kept set, its order and the values are those of oracle_rowtopk_fwd; a column
// index is stored in 16 bits, which every column of a row of D <= 65536 fits.
int oracle_rowtopk_fwd_idx16(const void* x, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                             uint16_t* idx_out, void* val_out, void* tau_out) {
    if (!idx_out || D > 65536u) return 1;
    std::vector<int32_t> idx(static_cast<size_t>(B) * k);
    const int rc = oracle_rowtopk_fwd(x, dtype, B, D, row_stride, k, idx.data(), val_out, tau_out);
    if (rc != 0) return rc;
    for (size_t o = 0; o < idx.size(); ++o) {
        if (idx[o] < 0 || idx[o] > 65535) return 3;
        idx_out[o] = static_cast<uint16_t>(idx[o]);
    }
    return 0;
}

// Backward through 16-bit indices: dval[b, j] = dy[b, idx[b, j]].
int oracle_rowtopk_bwd_idx16(const void* dy, int dtype, uint32_t B, uint32_t D, uint64_t row_stride, uint32_t k,
                             const uint16_t* idx, void* dval_out) {
    if (!dy || !idx || !dval_out || B == 0 || D == 0 || D > 65536u || k == 0 || k > D || row_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    for (uint32_t b = 0; b < B; ++b) {
        const unsigned char* row = static_cast<const unsigned char*>(dy) + es * row_stride * b;
        for (uint32_t j = 0; j < k; ++j) {
            const uint64_t o = static_cast<uint64_t>(b) * k + j;
            const uint32_t c = idx[o];
            if (c >= D) return 2;
            std::memcpy(static_cast<unsigned char*>(dval_out) + es * o, row + es * c, es);
        }
    }
    return 0;
}

// Receiver side for 16-bit indices: dense row = zeros with val[b, j] at column idx[b, j];
// a column >= D is skipped.
int oracle_rowscatter_idx16(const uint16_t* idx, const void* val, int dtype, uint32_t B, uint32_t D, uint32_t k,
                            void* out, uint64_t out_stride) {
    if (!idx || !val || !out || B == 0 || D == 0 || D > 65536u || k == 0 || out_stride < D) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return 1;
    const size_t es = elem_size(dtype);
    for (uint32_t b = 0; b < B; ++b) {
        unsigned char* row = static_cast<unsigned char*>(out) + es * out_stride * b;
        std::memset(row, 0, es * D);
        for (uint32_t j = 0; j < k; ++j) {
            const uint64_t o = static_cast<uint64_t>(b) * k + j;
            const uint32_t c = idx[o];
            if (c >= D) continue;
            std::memcpy(row + es * c, static_cast<const unsigned char*>(val) + es * o, es);
        }
    }
    return 0;
}

}  // extern "C"
