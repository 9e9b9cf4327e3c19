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
#include <atomic>
#include <cstdlib>
#include <numeric>
#include <thread>
#include <vector>

#include <immintrin.h>

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

int64_t popcount_and_generic(const uint64_t *a, const uint64_t *b, int64_t w)
{
    int64_t s = 0;
    for (int64_t i = 0; i < w; ++i) s += __builtin_popcountll(a[i] & b[i]);
    return s;
}

// Same count with 512-bit AND + per-lane population count, where the host CPU has them
// (checked once at run time: the library is built on one machine and run on another).
__attribute__((target("avx512f,avx512vpopcntdq")))
int64_t popcount_and_avx512(const uint64_t *a, const uint64_t *b, int64_t w)
{
    __m512i acc = _mm512_setzero_si512();
    int64_t i = 0;
    for (; i + 8 <= w; i += 8)
        acc = _mm512_add_epi64(acc, _mm512_popcnt_epi64(_mm512_and_si512(_mm512_loadu_si512(a + i), _mm512_loadu_si512(b + i))));
    int64_t s = _mm512_reduce_add_epi64(acc);
    for (; i < w; ++i) s += __builtin_popcountll(a[i] & b[i]);
    return s;
}

typedef int64_t (*popcount_and_fn)(const uint64_t *, const uint64_t *, int64_t);

// Threads of the candidate search that runs ahead of the greedy pass: the host's cores (at most
// 32), 1 for small inputs; the environment variable VBR_SA1_THREADS overrides the count.
int scan_threads(int64_t n_classes)
{
    if (const char *e = std::getenv("VBR_SA1_THREADS")) {
        const long v = std::strtol(e, nullptr, 10);
        if (v >= 1) return (int)std::min<long>(v, 256);
    }
    if (n_classes < 4096) return 1;
    const unsigned hw = std::thread::hardware_concurrency();
    return (int)std::max(1u, std::min(hw, 32u));
}

popcount_and_fn pick_popcount_and()
{
    __builtin_cpu_init();
    if (__builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512vpopcntdq")) return popcount_and_avx512;
    return popcount_and_generic;
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

    // Algorithm 2: one pass per seed over the later ungrouped classes in rising order, merging
    // where the condition of section 3.2 holds and OR-ing the merged pattern into the group's.
    const popcount_and_fn popcount_and = pick_popcount_and();
    // The similarity test (double)I / (double)U >= tau is monotone in I for a fixed U, so it is
    // tabulated once: need[U] = smallest I that passes (found with the very same division, so
    // the decisions are bit-identical), need[0] = 0 (two empty patterns are similar).
    std::vector<int32_t> need((size_t)KB + 1, 0);
    for (int64_t U = 1; U <= KB; ++U) {
        int64_t I = (int64_t)std::ceil(tau * (double)U);
        I = std::max<int64_t>(0, std::min<int64_t>(I, U));
        while (I > 0 && (double)(I - 1) / (double)U >= tau) --I;
        while (I <= U && !((double)I / (double)U >= tau)) ++I;      // I = U + 1: nothing passes
        need[U] = (int32_t)I;
    }
    std::vector<int32_t> group_of(std::max<int64_t>(NC, 1), -1);
    std::vector<uint64_t> P(W);
    int32_t G = 0;
    // the merge test for class j against the current pattern; updates the pattern on success
    int64_t sizeP = 0, lam_max = 0;
    auto try_merge = [&](int32_t j) -> bool {
        const int64_t lv = clen[j];
        if (sizeP == 0 && lv == 0) return true;            // both empty: similar, union 0 within any limit
        // |P & v| <= min and |P | v| >= max: if even min/max misses tau the exact ratio does too
        const int64_t lo = std::min(sizeP, lv), hi = std::max(sizeP, lv);
        if (lo < need[hi] || hi > lam_max) return false;
        const uint64_t *v = &cbits[(size_t)j * W];
        const int64_t I = popcount_and(P.data(), v, W);
        const int64_t U = sizeP + lv - I;
        if (I < need[U] || U > lam_max) return false;
        for (int64_t w = 0; w < W; ++w) P[w] |= v[w];
        sizeP = U;
        return true;
    };

    if (need[std::min<int64_t>(1, KB)] == 0) {
        // tau == 0: a class that shares nothing with the pattern can still pass the similarity
        // test, so every later class has to be looked at.  `active` = ungrouped classes, rising.
        std::vector<int32_t> active(NC), keep;
        std::iota(active.begin(), active.end(), 0);
        keep.reserve(NC);
        while (!active.empty()) {
            const int32_t seed = active[0];
            group_of[seed] = G;
            std::memcpy(P.data(), &cbits[(size_t)seed * W], (size_t)W * 8);
            sizeP = clen[seed];
            lam_max = (int64_t)std::floor((double)sizeP / (1.0 - 0.5 * tau));
            keep.clear();
            for (size_t t = 1; t < active.size(); ++t) {
                if (try_merge(active[t])) group_of[active[t]] = G;
                else keep.push_back(active[t]);
            }
            active.swap(keep);
            ++G;
        }
    } else {
        // tau > 0: a class can only pass if it shares a column block with the pattern (I >= 1).
        // An inverted index (block -> rising list of classes holding it) gives exactly those
        // classes: walking the lists of the pattern's blocks and counting how often a class shows
        // up yields |P & v| itself, with no bitset work.  Touched classes are flagged in a bitmap
        // and visited in rising order; when a merge adds blocks to the pattern, the tails of their
        // lists (classes above the current one) are counted in as well.  Every class that could
        // pass is met in the same order and with the same counts as in the full scan.
        std::vector<int64_t> inv_ptr((size_t)KB + 1, 0);
        for (int64_t c = 0; c < NC; ++c)
            for (int64_t w = 0; w < W; ++w)
                for (uint64_t x = cbits[(size_t)c * W + w]; x; x &= x - 1) inv_ptr[(w << 6) + __builtin_ctzll(x) + 1]++;
        for (int64_t b = 0; b < KB; ++b) inv_ptr[b + 1] += inv_ptr[b];
        std::vector<int32_t> inv((size_t)inv_ptr[KB]);
        {
            std::vector<int64_t> fill(inv_ptr.begin(), inv_ptr.end() - 1);
            for (int64_t c = 0; c < NC; ++c)
                for (int64_t w = 0; w < W; ++w)
                    for (uint64_t x = cbits[(size_t)c * W + w]; x; x &= x - 1) inv[fill[(w << 6) + __builtin_ctzll(x)]++] = (int32_t)c;
        }
        int32_t seed_done = -1;       // the seed being processed: classes up to it are never looked at again
        std::vector<int64_t> first(inv_ptr.begin(), inv_ptr.end() - 1);   // per block: first list entry above the seeds done
        std::vector<int32_t> cnt((size_t)std::max<int64_t>(NC, 1), 0);    // |P & v| of the touched classes
        const int64_t BW = (NC + 63) / 64 + 1;
        std::vector<uint64_t> touched((size_t)BW, 0);
        std::vector<uint64_t> before(W);
        // classes of block b above `above` are counted into cnt / touched
        auto count_list = [&](int64_t b, int32_t above) {
            int64_t &f = first[b];
            while (f < inv_ptr[b + 1] && inv[f] <= seed_done) ++f;         // seeds only rise: skipped for good
            const int64_t lo = above <= seed_done ? f : std::upper_bound(inv.begin() + f, inv.begin() + inv_ptr[b + 1], above) - inv.begin();
            for (int64_t e = lo; e < inv_ptr[b + 1]; ++e) {
                const int32_t c = inv[e];
                ++cnt[c];
                touched[c >> 6] |= 1ull << (c & 63);
            }
        };
        // The rest of a seed's pass from class `pos` on (pos itself is done), with the group's
        // pattern P as it stands: the classes above pos that share a block with P are counted,
        // visited in rising order, and merged where the condition holds; a merge counts in the tails
        // of the lists of the blocks it adds.
        auto scan_from = [&](int32_t pos) {
            for (int64_t w = 0; w < W; ++w)
                for (uint64_t x = P[w]; x; x &= x - 1) count_list((w << 6) + __builtin_ctzll(x), pos);
            for (int64_t tw = pos >> 6; tw < BW; ++tw) {
                while (touched[tw]) {
                    const int32_t j = (int32_t)((tw << 6) + __builtin_ctzll(touched[tw]));
                    touched[tw] &= touched[tw] - 1;
                    const int64_t I = cnt[j];
                    cnt[j] = 0;
                    if (group_of[j] != -1) continue;
                    const int64_t U = sizeP + clen[j] - I;
                    if (I < need[U] || U > lam_max) continue;
                    group_of[j] = G;                                        // merge: pattern <- OR
                    const uint64_t *v = &cbits[(size_t)j * W];
                    for (int64_t w = 0; w < W; ++w) { before[w] = P[w]; P[w] |= v[w]; }
                    sizeP = U;
                    for (int64_t w = 0; w < W; ++w)                         // tails of the lists of the new blocks
                        for (uint64_t x = P[w] & ~before[w]; x; x &= x - 1) {
                            const int64_t b = (w << 6) + __builtin_ctzll(x);
                            const int64_t lo = std::max(first[b], inv_ptr[b]);
                            for (int64_t e = std::upper_bound(inv.begin() + lo, inv.begin() + inv_ptr[b + 1], j) - inv.begin();
                                 e < inv_ptr[b + 1]; ++e) {
                                const int32_t c = inv[e];
                                ++cnt[c];
                                touched[c >> 6] |= 1ull << (c & 63);
                            }
                        }
                }
            }
        };
        // dense patterns make the lists long: when walking them costs more than comparing bitsets
        // with every later class, a seed does that instead (same decisions either way)
        auto lists_too_long = [&](const uint64_t *pat, int32_t seed) -> bool {
            int64_t list_work = 0;
            for (int64_t w = 0; w < W; ++w)
                for (uint64_t x = pat[w]; x; x &= x - 1) {
                    const int64_t b = (w << 6) + __builtin_ctzll(x);
                    list_work += inv_ptr[b + 1] - first[b];
                }
            return list_work > 4 * W * (NC - seed);
        };
        auto start_group = [&](int32_t seed) {
            group_of[seed] = G;
            std::memcpy(P.data(), &cbits[(size_t)seed * W], (size_t)W * 8);
            sizeP = clen[seed];
            lam_max = (int64_t)std::floor((double)sizeP / (1.0 - 0.5 * tau));
        };

        const int n_threads = scan_threads(NC);
        if (n_threads <= 1) {
            for (int32_t seed = 0; seed < NC; ++seed) {
                if (group_of[seed] != -1) continue;
                seed_done = seed;
                start_group(seed);
                if (lists_too_long(P.data(), seed)) {
                    for (int32_t j = seed + 1; j < NC; ++j)
                        if (group_of[j] == -1 && try_merge(j)) group_of[j] = G;
                } else {
                    scan_from(seed);
                }
                ++G;
            }
        } else {
            // Several threads.  The greedy pass itself stays sequential; what runs ahead of it, for a
            // batch of possible seeds at a time, is the search that costs the time when few rows
            // merge: for every class of the batch, the later classes that pass the merge test against
            // its OWN pattern (the group's pattern until its first merge), in rising order.  The
            // sequential pass then takes, for a class that is still ungrouped when its turn comes, the
            // first of those that is still ungrouped, merges it, and finishes that seed's scan from
            // there with the grown pattern as above.  Classes that do not pass against the seed's
            // own pattern cannot pass before the first merge, so the decisions, their order and the
            // groups are those of the one-thread pass.
            const int32_t batch = (int32_t)std::min<int64_t>(NC, (int64_t)n_threads * 512);
            std::vector<std::vector<int32_t>> passing((size_t)batch);
            std::vector<uint8_t> long_lists((size_t)batch, 0);
            for (int32_t b0 = 0; b0 < NC; b0 += batch) {
                const int32_t b1 = (int32_t)std::min<int64_t>(NC, (int64_t)b0 + batch);
                std::atomic<int32_t> next(b0);
                auto worker = [&]() {
                    std::vector<int32_t> my_cnt((size_t)NC, 0), hit;
                    for (;;) {
                        const int32_t c0 = next.fetch_add(16);
                        if (c0 >= b1) break;
                        for (int32_t seed = c0; seed < std::min(b1, c0 + 16); ++seed) {
                            std::vector<int32_t> &out = passing[(size_t)(seed - b0)];
                            out.clear();
                            long_lists[(size_t)(seed - b0)] = 0;
                            if (group_of[seed] != -1) continue;          // grouped before this batch began
                            const uint64_t *pat = &cbits[(size_t)seed * W];
                            if (lists_too_long(pat, seed)) { long_lists[(size_t)(seed - b0)] = 1; continue; }
                            hit.clear();
                            for (int64_t w = 0; w < W; ++w)
                                for (uint64_t x = pat[w]; x; x &= x - 1) {
                                    const int64_t b = (w << 6) + __builtin_ctzll(x);
                                    for (int64_t e = std::upper_bound(inv.begin() + inv_ptr[b], inv.begin() + inv_ptr[b + 1], seed) - inv.begin();
                                         e < inv_ptr[b + 1]; ++e) {
                                        const int32_t c = inv[e];
                                        if (my_cnt[c]++ == 0) hit.push_back(c);
                                    }
                                }
                            const int64_t sp = clen[seed];
                            const int64_t lim = (int64_t)std::floor((double)sp / (1.0 - 0.5 * tau));
                            for (const int32_t c : hit) {
                                const int64_t I = my_cnt[c];
                                my_cnt[c] = 0;
                                const int64_t U = sp + clen[c] - I;
                                if (I >= need[U] && U <= lim) out.push_back(c);
                            }
                            std::sort(out.begin(), out.end());
                        }
                    }
                };
                std::vector<std::thread> pool;
                for (int t = 1; t < n_threads; ++t) pool.emplace_back(worker);
                worker();
                for (std::thread &t : pool) t.join();

                for (int32_t seed = b0; seed < b1; ++seed) {
                    if (group_of[seed] != -1) continue;
                    seed_done = seed;
                    start_group(seed);
                    if (long_lists[(size_t)(seed - b0)]) {
                        for (int32_t j = seed + 1; j < NC; ++j)
                            if (group_of[j] == -1 && try_merge(j)) group_of[j] = G;
                    } else {
                        for (const int32_t j : passing[(size_t)(seed - b0)]) {
                            if (group_of[j] != -1) continue;
                            // the first class that passes and is still free: merge it, then go on from there
                            const uint64_t *v = &cbits[(size_t)j * W];
                            int64_t U = 0;
                            for (int64_t w = 0; w < W; ++w) { P[w] |= v[w]; U += __builtin_popcountll(P[w]); }
                            sizeP = U;
                            group_of[j] = G;
                            scan_from(j);
                            break;
                        }
                    }
                    ++G;
                }
            }
        }
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

namespace vbrk {
namespace {

// What the VBR matrix of a blocking would hold: per group the number of distinct column blocks
// its rows touch; a stored block of group g has height h_g.
void blocking_counts(const vbr_csr_t *csr, const int32_t *perm, const int32_t *row_groups, int32_t G,
                     int32_t col_block, int64_t *n_blocks, int64_t *stored_elems, int64_t *sum_heights)
{
    const int64_t KB = csr->n_cols / col_block;
    std::vector<int32_t> stamp((size_t)std::max<int64_t>(KB, 1), -1);
    int64_t nb = 0, stored = 0, sumh = 0;
    for (int32_t g = 0; g < G; ++g) {
        const int64_t h = row_groups[g + 1] - row_groups[g];
        int64_t cnt = 0;
        for (int64_t q = row_groups[g]; q < row_groups[g + 1]; ++q) {
            const int64_t r = perm[q];
            for (int64_t p = csr->row_ptr[r]; p < csr->row_ptr[r + 1]; ++p) {
                const int64_t j = csr->col_idx[p] / col_block;
                if (stamp[j] != g) { stamp[j] = g; ++cnt; }
            }
        }
        nb += cnt;
        stored += cnt * h * col_block;
        sumh += cnt * h;
    }
    *n_blocks = nb;
    *stored_elems = stored;
    *sum_heights = sumh;
}

}  // namespace
}  // namespace vbrk

extern "C" int sa1_blocking_curve(const vbr_csr_t *csr, int32_t col_block, const double *taus, int32_t n_taus,
                                  int64_t target_height, int64_t *n_groups, int64_t *n_blocks,
                                  int64_t *stored_elems, int64_t *sum_heights, int32_t *selected)
{
    if (!csr || !taus || n_taus <= 0 || col_block <= 0 || target_height <= 0) return VBR_EINVAL;
    for (int32_t i = 0; i < n_taus; ++i)
        if (!(taus[i] >= 0.0 && taus[i] <= 1.0)) return VBR_EINVAL;
    int rc = vbrk::validate_csr(csr, false);
    if (rc != VBR_OK) return rc;
    if (csr->n_cols % col_block != 0) return VBR_EINVAL;
    try {
        std::vector<int32_t> perm((size_t)csr->n_rows), rg((size_t)csr->n_rows + 1);
        int32_t best = 0;
        bool have = false;
        unsigned __int128 best_num = 0;    // |sum_heights - target * n_blocks| of the best so far
        int64_t best_den = 1;              // its n_blocks
        for (int32_t i = 0; i < n_taus; ++i) {
            int32_t G = 0;
            rc = vbrk::sa1_reorder_impl(csr, col_block, taus[i], perm.data(), rg.data(), &G);
            if (rc != VBR_OK) return rc;
            int64_t nb, stored, sumh;
            vbrk::blocking_counts(csr, perm.data(), rg.data(), G, col_block, &nb, &stored, &sumh);
            if (n_groups) n_groups[i] = G;
            if (n_blocks) n_blocks[i] = nb;
            if (stored_elems) stored_elems[i] = stored;
            if (sum_heights) sum_heights[i] = sumh;
            if (nb > 0) {
                // distance of the average block height from the target: |sumh / nb - target|
                const __int128 diff = (__int128)sumh - (__int128)target_height * nb;
                const unsigned __int128 num = (unsigned __int128)(diff < 0 ? -diff : diff);
                if (!have || num * (unsigned __int128)best_den < best_num * (unsigned __int128)nb) {
                    have = true;
                    best = i;
                    best_num = num;
                    best_den = nb;
                }
            }
        }
        if (selected) *selected = best;
        return VBR_OK;
    } catch (const std::bad_alloc &) {
        return VBR_ENOMEM;
    } catch (...) {
        return VBR_EINVAL;
    }
}
