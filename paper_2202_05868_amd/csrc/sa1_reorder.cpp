// 1-SA row reordering on the host: quotient rows as bitsets, grouping of identical quotient rows
// by hash + exact compare, greedy merge with pattern update under the two-step merge condition.
// Sections 3.1 and 3.2 of the paper (Eq. 4, Eq. 5, Algorithms 1 and 2, Theorem 1's condition).
// Integer work throughout; the only floating-point operations are one binary64 division per
// candidate (Jaccard >= tau) and one floor per seed (the merge limit).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include "vbr_host.h"

namespace vbrk {

int validate_csr(const vbr_csr_t *csr, bool need_vals)
{
    if (!csr) return VBR_EINVAL;
    if (csr->n_rows < 0 || csr->n_cols < 0 || csr->nnz < 0) return VBR_EINVAL;
    if (csr->n_rows > INT32_MAX - 1 || csr->n_cols > INT32_MAX - 1) return VBR_EINVAL;
    if (!csr->row_ptr) return VBR_EINVAL;
    if (csr->nnz > 0 && !csr->col_idx) return VBR_EINVAL;
    if (need_vals && csr->nnz > 0 && !csr->vals) return VBR_EINVAL;
    if (csr->dtype != VBR_F16 && csr->dtype != VBR_BF16) return VBR_EINVAL;
    const int64_t *rp = csr->row_ptr;
    if (rp[0] != 0 || rp[csr->n_rows] != csr->nnz) return VBR_EINVAL;
    for (int64_t i = 0; i < csr->n_rows; ++i) {
        if (rp[i + 1] < rp[i] || rp[i + 1] > csr->nnz) return VBR_EINVAL;
        int64_t last = -1;
        for (int64_t p = rp[i]; p < rp[i + 1]; ++p) {
            int64_t c = csr->col_idx[p];
            if (c <= last || c >= csr->n_cols) return VBR_EINVAL;   // unsorted, duplicate or out of range
            last = c;
        }
    }
    return VBR_OK;
}

namespace {

inline int64_t popcount_and(const uint64_t *a, const uint64_t *b, int64_t w)
{
    int64_t s = 0;
    for (int64_t i = 0; i < w; ++i) s += __builtin_popcountll(a[i] & b[i]);
    return s;
}

}  // namespace

int sa1_reorder_impl(const vbr_csr_t *csr, int32_t col_block, double tau, int32_t *perm,
                     int32_t *row_groups, int32_t *n_groups)
{
    const int64_t M = csr->n_rows;
    const int64_t KB = csr->n_cols / col_block;
    const int64_t W = std::max<int64_t>(1, (KB + 63) / 64);

    // Quotient rows (Eq. 4) as bitsets, with the hash of Eq. 5 (sum of the nonzero block
    // indices) and the row length, which the paper suggests to thin out collisions.
    std::vector<uint64_t> bits((size_t)M * W, 0);
    std::vector<uint64_t> hash(M, 0);
    std::vector<int32_t> len(M, 0);
    for (int64_t i = 0; i < M; ++i) {
        uint64_t *b = &bits[(size_t)i * W];
        int64_t last = -1;
        for (int64_t p = csr->row_ptr[i]; p < csr->row_ptr[i + 1]; ++p) {
            int64_t j = csr->col_idx[p] / col_block;
            if (j != last) {
                b[j >> 6] |= 1ull << (j & 63);
                hash[i] += (uint64_t)j;
                ++len[i];
                last = j;
            }
        }
    }

    // Algorithm 1 on the quotient rows: sort by (hash, length), then compare patterns exactly
    // inside each run of equal keys.  Rows of a run are visited in rising row order, so the
    // representative of a class is its smallest row.
    std::vector<int32_t> order(M);
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (hash[a] != hash[b]) return hash[a] < hash[b];
        if (len[a] != len[b]) return len[a] < len[b];
        return a < b;
    });
    std::vector<int32_t> rep_of(M, -1);   // row -> representative row of its class
    for (int64_t s = 0; s < M;) {
        int64_t e = s + 1;
        while (e < M && hash[order[e]] == hash[order[s]] && len[order[e]] == len[order[s]]) ++e;
        for (int64_t a = s; a < e; ++a) {
            int32_t ra = order[a];
            if (rep_of[ra] != -1) continue;
            rep_of[ra] = ra;
            const uint64_t *pa = &bits[(size_t)ra * W];
            for (int64_t b = a + 1; b < e; ++b) {
                int32_t rb = order[b];
                if (rep_of[rb] == -1 && std::memcmp(pa, &bits[(size_t)rb * W], (size_t)W * 8) == 0)
                    rep_of[rb] = ra;
            }
        }
        s = e;
    }
    // Classes in order of their smallest row: the order in which Algorithm 2 visits them.
    std::vector<int32_t> reps;
    for (int64_t i = 0; i < M; ++i)
        if (rep_of[i] == (int32_t)i) reps.push_back((int32_t)i);
    const int64_t NC = (int64_t)reps.size();
    std::vector<int32_t> class_index(M, -1);   // representative row -> class number
    std::vector<uint64_t> cbits((size_t)std::max<int64_t>(NC, 1) * W);
    std::vector<int32_t> clen(std::max<int64_t>(NC, 1));
    for (int64_t c = 0; c < NC; ++c) {
        class_index[reps[c]] = (int32_t)c;
        std::memcpy(&cbits[(size_t)c * W], &bits[(size_t)reps[c] * W], (size_t)W * 8);
        clen[c] = len[reps[c]];
    }
    bits.clear();
    bits.shrink_to_fit();

    // Algorithm 2.  `active` holds the classes not yet grouped, in rising order; one pass per
    // seed scans it once, merging where the condition of section 3.2 holds and OR-ing the
    // merged pattern into the group's pattern.
    std::vector<int32_t> group_of(std::max<int64_t>(NC, 1), -1);
    std::vector<int32_t> active(NC), keep;
    std::iota(active.begin(), active.end(), 0);
    keep.reserve(NC);
    std::vector<uint64_t> P(W);
    int32_t G = 0;
    while (!active.empty()) {
        const int32_t seed = active[0];
        group_of[seed] = G;
        std::memcpy(P.data(), &cbits[(size_t)seed * W], (size_t)W * 8);
        int64_t sizeP = clen[seed];
        const int64_t lambda0 = sizeP;
        const int64_t lam_max = (int64_t)std::floor((double)lambda0 / (1.0 - 0.5 * tau));
        keep.clear();
        for (size_t t = 1; t < active.size(); ++t) {
            const int32_t j = active[t];
            const int64_t lv = clen[j];
            bool merge = false;
            if (sizeP == 0 && lv == 0) {
                merge = true;                         // both empty: similar, union 0 within any limit
            } else {
                // |P & v| <= min and |P | v| >= max: if even min/max misses tau the exact ratio does too
                const int64_t lo = std::min(sizeP, lv), hi = std::max(sizeP, lv);
                if ((double)lo / (double)hi >= tau && hi <= lam_max) {
                    const uint64_t *v = &cbits[(size_t)j * W];
                    const int64_t I = popcount_and(P.data(), v, W);
                    const int64_t U = sizeP + lv - I;
                    if ((double)I / (double)U >= tau && U <= lam_max) {
                        merge = true;
                        for (int64_t w = 0; w < W; ++w) P[w] |= v[w];
                        sizeP = U;
                    }
                }
            }
            if (merge) group_of[j] = G;
            else keep.push_back(j);
        }
        active.swap(keep);
        ++G;
    }

    // Rows sorted by group, stable in the row index; groups are already numbered in seed order.
    std::vector<int64_t> start((size_t)G + 1, 0);
    for (int64_t i = 0; i < M; ++i) start[group_of[class_index[rep_of[i]]] + 1]++;
    for (int32_t g = 0; g < G; ++g) start[g + 1] += start[g];
    for (int32_t g = 0; g <= G; ++g) row_groups[g] = (int32_t)start[g];
    for (int64_t i = 0; i < M; ++i) perm[start[group_of[class_index[rep_of[i]]]]++] = (int32_t)i;
    *n_groups = G;
    return VBR_OK;
}

}  // namespace vbrk

extern "C" int sa1_reorder(const vbr_csr_t *csr, int32_t col_block, double tau, int32_t *perm,
                           int32_t *row_groups, int32_t *n_groups)
{
    if (!csr || !perm || !row_groups || !n_groups) return VBR_EINVAL;
    if (col_block <= 0 || !(tau >= 0.0 && tau <= 1.0)) return VBR_EINVAL;
    int rc = vbrk::validate_csr(csr, false);
    if (rc != VBR_OK) return rc;
    if (csr->n_cols % col_block != 0) return VBR_EINVAL;
    try {
        return vbrk::sa1_reorder_impl(csr, col_block, tau, perm, row_groups, n_groups);
    } catch (const std::bad_alloc &) {
        return VBR_ENOMEM;
    } catch (...) {
        return VBR_EINVAL;
    }
}
