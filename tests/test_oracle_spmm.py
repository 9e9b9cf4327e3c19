"""Pins for the oracle's C = A.B (CPU only): brute-force dense products, identity right-hand
sides, a single dense block (plain GEMM), row subsets, and the exactness of the 16-bit decode."""
import numpy as np

import oracle
from paper_2202_05868_amd import synth
from helpers import random_csr


def dense_f64(csr):
    return oracle.bits_to_f64(synth.dense_bits(csr), csr["dtype"])


def test_decode_of_16_bit_patterns_is_exact():
    # fp16: 1.0 = 0x3C00, -2.0 = 0xC000, smallest subnormal 2^-24 = 0x0001, 65504 = 0x7BFF
    bits = np.array([0x3C00, 0xC000, 0x0001, 0x7BFF, 0x0000, 0x8000], dtype=np.uint16)
    got = oracle.bits_to_f64(bits, "f16")
    assert np.array_equal(got, np.array([1.0, -2.0, 2.0 ** -24, 65504.0, 0.0, -0.0]))
    # bf16: 1.0 = 0x3F80, -2.0 = 0xC000, 2^-126 = 0x0080, 3.140625 = 0x4049
    bits = np.array([0x3F80, 0xC000, 0x0080, 0x4049], dtype=np.uint16)
    got = oracle.bits_to_f64(bits, "bf16")
    assert np.array_equal(got, np.array([1.0, -2.0, 2.0 ** -126, 3.140625]))


def test_rounding_to_storage_types_is_nearest_even():
    x = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)
    h = oracle.bits_to_f64(synth.to_bits(x[:2], "f16"), "f16")        # ties: to even mantissa
    assert np.array_equal(h, [1.0, 1.0 + 2.0 ** -9])
    b = oracle.bits_to_f64(synth.to_bits(x[2:], "bf16"), "bf16")
    assert np.array_equal(b, [1.0, 1.0 + 2.0 ** -6])


def test_matches_brute_force_dense_product():
    rng = np.random.default_rng(1)
    for dtype in ("f16", "bf16"):
        for (m, k, n, d) in [(17, 23, 9, 0.3), (64, 48, 40, 0.05), (5, 7, 3, 1.0), (33, 16, 8, 0.0)]:
            csr = random_csr(rng, m, k, d, dtype=dtype)
            b = synth.dense_rhs(rng, k, n, dtype)
            c, s = oracle.spmm(csr, b)
            a64 = dense_f64(csr)
            b64 = oracle.bits_to_f64(b, dtype)
            c_ref = a64 @ b64
            s_ref = np.abs(a64) @ np.abs(b64)
            assert np.allclose(c, c_ref, rtol=0, atol=1e-12 * (1 + s_ref.max(initial=0)))
            assert np.allclose(s, s_ref, rtol=1e-13, atol=0)
            # every product of two 16-bit values is exact in binary64, and so are short sums:
            # the sequential sum may differ from the library's only in the last bits
            assert np.all(np.abs(c - c_ref) <= 1e-13 * s_ref + 1e-300)


def test_identity_right_hand_side_returns_the_matrix():
    rng = np.random.default_rng(2)
    csr = random_csr(rng, 40, 24, 0.2)
    eye = synth.to_bits(np.eye(24, dtype=np.float32), "f16")
    c, s = oracle.spmm(csr, eye)
    assert np.array_equal(c, dense_f64(csr))
    assert np.array_equal(s, np.abs(dense_f64(csr)))


def test_single_dense_block_is_a_plain_gemm():
    rng = np.random.default_rng(3)
    csr = random_csr(rng, 12, 20, 1.0)
    b = synth.dense_rhs(rng, 20, 12, "f16")
    c, _ = oracle.spmm(csr, b)
    a64, b64 = dense_f64(csr), oracle.bits_to_f64(b, "f16")
    assert np.allclose(c, a64 @ b64, rtol=0, atol=1e-12)
    # non-square on purpose: a transposed operand or swapped index cannot produce this shape/value
    assert c.shape == (12, 12) and not np.allclose(c, (a64 @ b64).T, atol=1e-3)


def test_row_subset_equals_rows_of_the_full_product():
    rng = np.random.default_rng(4)
    csr = random_csr(rng, 50, 32, 0.15)
    b = synth.dense_rhs(rng, 32, 16, "f16")
    c, s = oracle.spmm(csr, b)
    rows = np.array([49, 0, 7, 7, 31])
    c2, s2 = oracle.spmm(csr, b, rows=rows)
    assert np.array_equal(c2, c[rows]) and np.array_equal(s2, s[rows])
    c3, none = oracle.spmm(csr, b, rows=rows, with_bound=False)
    assert none is None and np.array_equal(c3, c[rows])


def test_product_does_not_depend_on_the_row_order_of_the_input():
    rng = np.random.default_rng(6)
    csr = random_csr(rng, 30, 16, 0.3)
    b = synth.dense_rhs(rng, 16, 8, "f16")
    c, _ = oracle.spmm(csr, b)
    order = rng.permutation(30)
    c_p, _ = oracle.spmm(synth.permute_rows(csr, order), b)
    assert np.array_equal(c_p, c[order])


def test_landscape_generator_draws_what_section_4_1_states():
    # input generator only (no method arithmetic): theta of ALL blocks flagged, rho of the entries
    # of each flagged block kept, rows scrambled
    from paper_2202_05868_amd import synth
    rng = np.random.default_rng(5)
    n, delta, theta, rho = 512, 32, 0.2, 0.1
    a = synth.landscape(rng, n, delta, theta, rho, scramble=False)
    g = n // delta
    rows = np.repeat(np.arange(n), np.diff(a["row_ptr"]))
    blk = (rows // delta) * g + a["col_idx"] // delta
    ids, counts = np.unique(blk, return_counts=True)
    assert ids.size == round(theta * g * g)
    assert np.all(counts == round(rho * delta * delta))
    b = synth.landscape(np.random.default_rng(5), n, delta, theta, rho)      # same draw, rows scrambled
    assert b["nnz"] == a["nnz"] and sorted(np.diff(b["row_ptr"]).tolist()) == sorted(np.diff(a["row_ptr"]).tolist())
