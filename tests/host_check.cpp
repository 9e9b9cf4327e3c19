// Host-side check program for the sanitizer build: the library's host units (1-SA, VBR build, block
// unpacking, blocking curve, bounds audit) linked with the C oracle into one executable compiled with
// -fsanitize=address,undefined, and driven over seeded random matrices.  Every case compares the
// library with the oracle bit for bit and runs the audit of everything the kernels would index, so
// that an out-of-bounds access, an overflow or a leak in 500 lines of hand index arithmetic shows up
// on the CPU.  Test infrastructure: built and run by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "vbr_spmm.h"

extern "C" {
int oracle_sa1(int64_t n_rows, int64_t n_cols, const int64_t *row_ptr, const int32_t *col_idx, int32_t col_block,
               double tau, int32_t similarity_only, int32_t *perm, int32_t *row_groups, int32_t *n_groups);
int oracle_vbr_index(int64_t n_rows, int64_t n_cols, const int64_t *row_ptr, const int32_t *col_idx, int32_t col_block,
                     const int32_t *perm, const int32_t *row_groups, int32_t n_groups, int64_t *blk_ptr,
                     int32_t *blk_col, int64_t *blk_off, int64_t *n_blocks);
}

namespace {

struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 1) {}
    uint64_t next() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
    double uni() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
    int64_t below(int64_t n) { return (int64_t)(uni() * (double)n); }
};

struct Csr {
    int64_t m = 0, k = 0;
    std::vector<int64_t> row_ptr;
    std::vector<int32_t> col;
    std::vector<uint16_t> val;
    vbr_csr_t view() const
    {
        vbr_csr_t c;
        c.n_rows = m; c.n_cols = k; c.nnz = (int64_t)col.size();
        c.row_ptr = row_ptr.data(); c.col_idx = col.data(); c.vals = val.data(); c.dtype = VBR_F16;
        return c;
    }
};

// rows drawn from `n_base` base patterns over the column blocks, each with a little noise, so that
// identical rows, merges, refusals and the size limit all occur
Csr make(Rng &rng, int64_t m, int64_t kb, int col_block, double density, int n_base)
{
    Csr a;
    a.m = m; a.k = kb * col_block;
    std::vector<std::vector<uint8_t>> base((size_t)n_base, std::vector<uint8_t>((size_t)kb, 0));
    for (auto &b : base)
        for (auto &x : b) x = rng.uni() < density;
    a.row_ptr.push_back(0);
    for (int64_t i = 0; i < m; ++i) {
        const auto &b = base[(size_t)rng.below(n_base)];
        for (int64_t j = 0; j < kb; ++j) {
            const bool on = b[(size_t)j] != (rng.uni() < density * 0.1);
            if (!on) continue;
            for (int c = 0; c < col_block; ++c)
                if (c == 0 || rng.uni() < 0.4) {
                    a.col.push_back((int32_t)(j * col_block + c));
                    a.val.push_back((uint16_t)(1 + rng.below(0x7bff)));
                }
        }
        a.row_ptr.push_back((int64_t)a.col.size());
    }
    return a;
}

int g_cases = 0;
#define REQUIRE(cond) do { if (!(cond)) { std::fprintf(stderr, "host_check: %s failed at line %d (case %d)\n", #cond, __LINE__, g_cases); std::exit(1); } } while (0)

void check_matrix(const Csr &a, int col_block, double tau, bool all_blocks)
{
    ++g_cases;
    const vbr_csr_t c = a.view();
    std::vector<int32_t> perm((size_t)a.m), rg((size_t)a.m + 1), perm0((size_t)a.m), rg0((size_t)a.m + 1);
    int32_t G = 0, G0 = 0;
    REQUIRE(sa1_reorder(&c, col_block, tau, perm.data(), rg.data(), &G) == VBR_OK);
    REQUIRE(oracle_sa1(a.m, a.k, c.row_ptr, c.col_idx, col_block, tau, 0, perm0.data(), rg0.data(), &G0) == 0);
    REQUIRE(G == G0);
    REQUIRE(std::memcmp(perm.data(), perm0.data(), (size_t)a.m * 4) == 0);
    REQUIRE(std::memcmp(rg.data(), rg0.data(), ((size_t)G + 1) * 4) == 0);

    vbr_t *v = nullptr;
    REQUIRE(vbr_build(&c, perm.data(), rg.data(), G, col_block, &v) == VBR_OK);
    REQUIRE(vbr_audit(v) == VBR_OK);
    REQUIRE(vbr_device_bytes(v) >= 256 && vbr_device_bytes(v) % 256 == 0);
    const int32_t *vrg, *vperm, *bcol;
    const int64_t *bptr, *boff;
    int64_t ng, nb, stored;
    REQUIRE(vbr_get_index(v, &vrg, &vperm, &bptr, &bcol, &boff, &ng, &nb, &stored) == VBR_OK);
    const int64_t cap = c.nnz + 1;
    std::vector<int64_t> bptr0((size_t)G + 1), boff0((size_t)cap + 1);
    std::vector<int32_t> bcol0((size_t)cap);
    int64_t nb0 = 0;
    REQUIRE(oracle_vbr_index(a.m, a.k, c.row_ptr, c.col_idx, col_block, perm.data(), rg.data(), G, bptr0.data(),
                             bcol0.data(), boff0.data(), &nb0) == 0);
    REQUIRE(nb == nb0 && ng == G);
    REQUIRE(std::memcmp(bptr, bptr0.data(), ((size_t)G + 1) * 8) == 0);
    REQUIRE(std::memcmp(bcol, bcol0.data(), (size_t)nb * 4) == 0);
    REQUIRE(std::memcmp(boff, boff0.data(), ((size_t)nb + 1) * 8) == 0);
    REQUIRE(stored == boff0[(size_t)nb]);
    // stored blocks read back out of the packed layout = the zero-filled windows of the matrix
    std::vector<uint16_t> got, want;
    for (int32_t g = 0; g < G; ++g) {
        const int64_t h = rg[(size_t)g + 1] - rg[(size_t)g];
        for (int64_t b = bptr[g]; b < bptr[g + 1]; ++b) {
            if (!all_blocks && (b % 7) != 0) continue;
            got.assign((size_t)(h * col_block), 0xffff);
            want.assign((size_t)(h * col_block), 0);
            REQUIRE(vbr_unpack_block(v, b, got.data()) == VBR_OK);
            for (int64_t t = 0; t < h; ++t) {
                const int64_t r = perm[(size_t)(rg[(size_t)g] + t)];
                for (int64_t p = c.row_ptr[r]; p < c.row_ptr[r + 1]; ++p)
                    if (c.col_idx[p] / col_block == bcol[b]) want[(size_t)(t * col_block + c.col_idx[p] % col_block)] = a.val[(size_t)p];
            }
            REQUIRE(got == want);
        }
    }
    int32_t n_launch = 0, kinds[VBR_MAX_LAUNCHES];
    int64_t tiles[VBR_MAX_LAUNCHES], wgs[VBR_MAX_LAUNCHES];
    REQUIRE(vbr_get_launches(v, 264, &n_launch, kinds, tiles, wgs) == VBR_OK && n_launch <= VBR_MAX_LAUNCHES);
    vbr_free(v);
}

}  // namespace

int main()
{
    Rng rng(12345);
    const double taus[] = {0.0, 0.3, 0.6, 1.0};
    // small matrices, every block width class (narrow gather path, granules of 8, 16, 32)
    for (int col_block : {1, 3, 8, 16, 32, 64})
        for (int trial = 0; trial < 4; ++trial) {
            const Csr a = make(rng, 1 + rng.below(400), 1 + rng.below(40), col_block, 0.05 + 0.3 * rng.uni(), 1 + (int)rng.below(30));
            for (double tau : taus) check_matrix(a, col_block, tau, true);
        }
    // thousands of short groups: the panel packing; tall groups beside them
    {
        const Csr a = make(rng, 6000, 40, 8, 0.08, 3000);
        check_matrix(a, 8, 0.9, false);
        const Csr b = make(rng, 5000, 24, 16, 0.15, 40);
        check_matrix(b, 16, 0.5, false);
        check_matrix(b, 16, 1.0, false);
    }
    // the candidate search on several threads against the same oracle
    {
        setenv("VBR_SA1_THREADS", "3", 1);
        const Csr a = make(rng, 5000, 300, 2, 0.02, 400);
        for (double tau : {0.2, 0.5, 0.9}) check_matrix(a, 2, tau, false);
        unsetenv("VBR_SA1_THREADS");
    }
    // blocking curve and error paths
    {
        const Csr a = make(rng, 300, 20, 4, 0.2, 12);
        const vbr_csr_t c = a.view();
        const double ts[] = {0.1, 0.5, 1.0};
        int64_t g[3], nb[3], st[3], sh[3];
        int32_t sel = -1;
        REQUIRE(sa1_blocking_curve(&c, 4, ts, 3, 8, g, nb, st, sh, &sel) == VBR_OK && sel >= 0 && sel < 3);
        REQUIRE(sa1_blocking_curve(&c, 4, ts, 3, 0, g, nb, st, sh, &sel) == VBR_EINVAL);
        std::vector<int32_t> perm((size_t)a.m, 0), rg = {0, (int32_t)a.m};
        vbr_t *v = nullptr;
        REQUIRE(vbr_build(&c, perm.data(), rg.data(), 1, 4, &v) == VBR_EINVAL && v == nullptr);   // not a bijection
        REQUIRE(sa1_reorder(&c, 3, 0.5, perm.data(), rg.data(), &sel) == VBR_EINVAL);            // 80 % 3 != 0
        REQUIRE(vbr_audit(nullptr) == VBR_EINVAL);
        ++g_cases;
    }
    std::printf("host_check ok: %d cases\n", g_cases);
    return 0;
}
