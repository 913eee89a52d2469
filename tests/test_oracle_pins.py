"""Pins of the CPU oracle to facts the paper and the mathematics fix.

None of these tests compares the oracle with itself or with the HIP path: each
checks it against a closed form, a library routine, a brute-force restatement of
the prose definition, a hand-computed example, or an error bound from the paper.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def heap_slot(t, i):
    """Slot of threshold v^t_i (both 1-based) in the 16-float array of one tree."""
    return (1 << (t - 1)) - 1 + (i - 1)


# ---------------------------------------------------------------------------
# Algorithm 1 (Section 4.1)
# ---------------------------------------------------------------------------

class Node:
    """Explicit binary tree built from the prose of Section 4.1: go left if the
    value is below the node's threshold, right otherwise; leaves are the hash
    buckets, numbered left to right."""

    def __init__(self, level, lo_leaf, hi_leaf, thr_of):
        self.level = level
        if hi_leaf - lo_leaf == 1:
            self.leaf = lo_leaf
            return
        self.leaf = None
        mid = (lo_leaf + hi_leaf) // 2
        # position of this node within its level = lo_leaf / (leaves per node)
        width = hi_leaf - lo_leaf
        self.thr = thr_of(level, lo_leaf // width + 1)
        self.left = Node(level + 1, lo_leaf, mid, thr_of)
        self.right = Node(level + 1, mid, hi_leaf, thr_of)

    def walk(self, x, dims):
        if self.leaf is not None:
            return self.leaf
        below = x[dims[self.level - 1]] < self.thr
        return (self.left if below else self.right).walk(x, dims)


def test_hash_matches_pointer_tree_brute_force():
    rng = np.random.default_rng(1)
    for trial in range(20):
        D = 9
        dims = rng.choice(D, size=4, replace=trial % 2 == 0).astype(np.int32)
        v = rng.standard_normal(16).astype(np.float32)
        root = Node(1, 0, 16, lambda t, i: v[heap_slot(t, i)])
        X = rng.standard_normal((200, D)).astype(np.float32)
        # put some values exactly on thresholds
        X[:40, dims[trial % 4]] = v[rng.integers(0, 15, size=40)]
        for x in X:
            assert oracle.hash_row(x, dims, v) == root.walk(x, dims) + 1


def test_widening_is_exact_for_every_bit_pattern():
    """binary16, bfloat16 and bytes all widen to fp32 without rounding.  binary16 against
    NumPy's conversion (library routine) on all 65536 patterns and against values fixed by
    the format; bfloat16 against "the upper half of an fp32" spelled out with struct."""
    import struct
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, "f16")
    ref = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert nan.sum() == 2046 and (np.isnan(got) == nan).all()
    assert (got.view(np.uint32)[~nan] == ref.view(np.uint32)[~nan]).all()      # also the sign of zero
    fixed = {0x3C00: 1.0, 0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24, 0x0400: 2.0 ** -14,
             0x7BFF: 65504.0, 0xC000: -2.0, 0x3555: 0.333251953125}
    for h, val in fixed.items():
        assert got[h] == np.float32(val)
    assert got[0x7C00] == np.inf and got[0xFC00] == -np.inf and np.signbit(got[0x8000]) and got[0x8000] == 0
    got = oracle.widen(bits, "bf16")
    for b in list(range(0, 65536, 97)) + [0x3F80, 0x4049, 0x0001, 0x8000, 0x7F80, 0xFF80, 0x7FC0]:
        want = struct.unpack("<f", struct.pack("<I", b << 16))[0]
        assert (np.isnan(want) and np.isnan(got[b])) or (got[b] == want and np.signbit(got[b]) == np.signbit(want))
    assert got[0x3F80] == 1.0 and got[0x4049] == 3.140625 and got[0x0001] == 2.0 ** -133
    assert (oracle.widen(np.arange(256, dtype=np.uint8), "u8") == np.arange(256)).all()


def test_typed_and_column_major_encode_by_brute_force():
    """g on narrow inputs and on inputs stored by columns (Section 4.1; Appendix E.6) against the
    pointer tree walked on Python floats of the same values."""
    rng = np.random.default_rng(11)
    N, D, Cc = 120, 12, 5
    sd = rng.integers(0, D, size=(Cc, 4)).astype(np.int32)
    for dtype in ("f32", "f16", "bf16", "u8"):
        if dtype == "u8":
            A = rng.integers(0, 256, size=(N, D)).astype(np.uint8)
            values = A.astype(np.float64)
            th = (rng.integers(0, 256, size=(Cc, 16)) + rng.choice([0.0, 0.5], size=(Cc, 16))).astype(np.float32)
        elif dtype == "bf16":
            A = (rng.standard_normal((N, D)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
            values = (A.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            th = rng.standard_normal((Cc, 16)).astype(np.float32)
        else:
            A = rng.standard_normal((N, D)).astype(np.float16 if dtype == "f16" else np.float32)
            values = A.astype(np.float64)
            th = rng.standard_normal((Cc, 16)).astype(np.float32)
        # thresholds that coincide with data values: equal goes right
        for c in range(Cc):
            th[c, :4] = values[rng.integers(0, N, size=4), sd[c, 0]].astype(np.float32)
        expect = np.empty((N, Cc), dtype=np.uint8)
        for c in range(Cc):
            root = Node(1, 0, 16, lambda t, i: float(th[c, heap_slot(t, i)]))
            for n in range(N):
                expect[n, c] = root.walk(values[n], sd[c])
        assert (oracle.encode_typed(A, dtype, False, sd, th) == expect).all(), dtype
        assert (oracle.encode_typed(np.ascontiguousarray(A.T), dtype, True, sd, th) == expect).all(), dtype
        # padded leading dimensions
        Ap = np.zeros((N, D + 3), dtype=A.dtype); Ap[:, :D] = A
        assert (oracle.encode_typed(Ap, dtype, False, sd, th)[:, :] == expect).all()


def test_hash_closed_form_when_levels_share_one_threshold():
    # If every node of level t has the same threshold theta_t, the four tests are
    # independent and the leaf is the 4-bit number they spell, level 1 first.
    rng = np.random.default_rng(2)
    theta = np.array([0.3, -0.2, 0.9, 0.0], dtype=np.float32)
    v = np.zeros(16, dtype=np.float32)
    for t in range(1, 5):
        for i in range(1, (1 << (t - 1)) + 1):
            v[heap_slot(t, i)] = theta[t - 1]
    dims = np.array([5, 1, 7, 2], dtype=np.int32)
    X = rng.standard_normal((500, 8)).astype(np.float32)
    bits = (X[:, dims] >= theta).astype(int)
    expect = bits[:, 0] * 8 + bits[:, 1] * 4 + bits[:, 2] * 2 + bits[:, 3]
    sd = dims[None, :]
    codes = oracle.encode(X, sd, v[None, :])
    assert (codes[:, 0] == expect).all()
    # all 16 leaves are reached
    assert set(expect.tolist()) == set(range(16))


def test_hash_reduces_to_searchsorted_on_one_dimension():
    # Four levels on the same coordinate with the 15 thresholds laid out as a
    # balanced search tree over sorted values s: the leaf is the number of s <= x.
    rng = np.random.default_rng(3)
    s = np.sort(rng.standard_normal(15)).astype(np.float32)
    v = np.zeros(16, dtype=np.float32)
    for t in range(1, 5):
        n_nodes = 1 << (t - 1)
        step = 16 // n_nodes
        for i in range(1, n_nodes + 1):
            v[heap_slot(t, i)] = s[(i - 1) * step + step // 2 - 1]
    x = np.concatenate([rng.standard_normal(1000).astype(np.float32) * 2, s])  # includes x == threshold
    X = np.zeros((x.size, 3), dtype=np.float32)
    X[:, 1] = x
    codes = oracle.encode(X, np.array([[1, 1, 1, 1]], dtype=np.int32), v[None, :])
    assert (codes[:, 0] == np.searchsorted(s, x, side="right")).all()


def test_hash_boundaries():
    v = np.zeros(16, dtype=np.float32)      # every threshold +0.0
    j = np.array([0, 0, 0, 0], dtype=np.int32)
    f = lambda val: oracle.hash_row(np.array([val], dtype=np.float32), j, v)
    assert f(0.0) == 16          # equal goes right at every level
    assert f(-0.0) == 16         # -0.0 >= +0.0 is true
    assert f(np.nan) == 1        # NaN compares false: left at every level
    assert f(-1e-30) == 1
    assert f(np.inf) == 16 and f(-np.inf) == 1
    vn = np.full(16, np.nan, dtype=np.float32)
    assert oracle.hash_row(np.array([1.0], dtype=np.float32), j, vn) == 1


def test_codes_use_four_bits_and_fifteen_thresholds():
    # Proof of Lemma F.1: a tree has 4 split indices and 15 split values; changing
    # the 16th slot must not change any code.
    rng = np.random.default_rng(4)
    X = rng.standard_normal((4000, 6)).astype(np.float32)
    sd = np.stack([rng.permutation(6)[:4] for _ in range(3)]).astype(np.int32)   # distinct per tree
    th = (0.3 * rng.standard_normal((3, 16))).astype(np.float32)
    c1 = oracle.encode(X, sd, th)
    th2 = th.copy(); th2[:, 15] = 1e9
    assert (oracle.encode(X, sd, th2) == c1).all()
    assert c1.max() <= 15
    for slot in range(15):       # ... and every one of the 15 does matter
        th3 = th.copy(); th3[:, slot] += 0.7
        assert (oracle.encode(X, sd, th3) != c1).any()


def test_pack_layout():
    codes = np.array([[1, 2, 3], [15, 0, 9]], dtype=np.uint8)
    assert oracle.pack(codes).tolist() == [[0x21, 0x03], [0x0F, 0x09]]
    rng = np.random.default_rng(5)
    c = rng.integers(0, 16, size=(50, 8)).astype(np.uint8)
    p = oracle.pack(c)
    assert p.shape == (50, 4)
    assert ((p & 15) == c[:, 0::2]).all() and ((p >> 4) == c[:, 1::2]).all()


# ---------------------------------------------------------------------------
# one-hot matrix G: the paper's printed example (Section 4.3)
# ---------------------------------------------------------------------------

def _one_hot_rows(codes, n_protos=16):
    """One-hot rows built with a library identity matrix (a checker that is not the oracle's)."""
    codes = np.asarray(codes)
    return np.eye(n_protos)[codes].reshape(codes.shape[0], codes.shape[1] * n_protos)


def test_one_hot_printed_example():
    lines = [l for l in open(os.path.join(GOLD, "onehot_example.txt")) if not l.startswith("#")]
    Kk, Cc = map(int, lines[0].split())
    assign = np.array(lines[1].split(), dtype=int)
    row = np.array(lines[2].split(), dtype=float)
    G = oracle.one_hot((assign - 1)[None, :].astype(np.uint8), n_protos=Kk)
    assert G.shape == (1, Kk * Cc) and (G[0] == row).all()
    assert (_one_hot_rows((assign - 1)[None, :], Kk)[0] == row).all()
    # and on random codes the oracle's G is the library construction
    codes = np.random.default_rng(0).integers(0, 16, size=(50, 5)).astype(np.uint8)
    assert (oracle.one_hot(codes) == _one_hot_rows(codes)).all()


# ---------------------------------------------------------------------------
# tables h(B) (Section 3) and the exact-table identity (proof of Lemma F.5)
# ---------------------------------------------------------------------------

def _small_problem(seed, N=64, D=12, M=5, Cc=3):
    rng = np.random.default_rng(seed)
    P = rng.standard_normal((Cc, 16, D)).astype(np.float32)
    B = rng.standard_normal((D, M)).astype(np.float32)
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    return P, B, codes


def test_float_tables_equal_library_contraction():
    P, B, _ = _small_problem(6)
    T = oracle.build_luts_f64(P, B)
    ref = np.einsum("ckd,dm->ckm", P.astype(np.float64), B.astype(np.float64))
    np.testing.assert_allclose(T, ref, rtol=1e-13, atol=1e-13)
    # a transposed B would fail: B is not square here and P B != P B^T
    assert T.shape == (3, 16, 5)


def test_sum_of_exact_tables_is_reconstruction_times_B():
    P, B, codes = _small_problem(7)
    T = oracle.build_luts_f64(P, B)
    got = oracle.scan_f64(oracle.pack(codes), 3, T)
    G = _one_hot_rows(codes)
    A_hat = G @ P.reshape(48, -1).astype(np.float64)      # rows rebuilt from prototypes
    np.testing.assert_allclose(got, A_hat @ B.astype(np.float64), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# 8-bit quantisation (Section 3; Appendix A)
# ---------------------------------------------------------------------------

def _table(vals):
    """One codebook, one column; 16 entries, the given ones then repeats of the first."""
    t = np.full(16, vals[0], dtype=np.float64)
    t[:len(vals)] = vals
    return t.reshape(1, 16, 1)


def test_quantize_hand_example():
    luts, scale, offset, l, delta = oracle.quantize_luts(_table([0, 1, 2.5, 100]))
    assert l[0] == 1 and scale[0] == 0.5 and offset[0] == 0.0
    assert luts[0, :4, 0].tolist() == [0, 2, 5, 200]
    # shifted table: same bytes, offset moves
    luts2, scale2, offset2, _, _ = oracle.quantize_luts(_table([0, 1, 2.5, 100]) - 7.25)
    assert (luts2 == luts).all() and scale2[0] == 0.5 and offset2[0] == -7.25


def test_quantize_rounds_half_to_even():
    luts, scale, _, l, _ = oracle.quantize_luts(_table([0, 0.5, 1.5, 2.5, 3.5, 255]))
    assert l[0] == 0 and scale[0] == 1.0
    assert luts[0, :6, 0].tolist() == [0, 0, 2, 2, 4, 255]


@pytest.mark.parametrize("r,l_expect", [(255.0, 0), (np.nextafter(255.0, 300), -1), (127.5, 1),
                                        (np.nextafter(127.5, 200), 0), (1.0, 7), (256.0, -1),
                                        (1e-3, 17), (3e5, -11)])
def test_scale_exponent_is_largest_power_of_two_that_fits(r, l_expect):
    _, scale, _, l, _ = oracle.quantize_luts(_table([0, r]))
    assert l[0] == l_expect
    assert r * 2.0 ** l[0] <= 255.0 < r * 2.0 ** (l[0] + 1)
    assert scale[0] == np.float32(2.0 ** -l[0])


def test_scale_is_set_by_the_widest_table_of_the_column():
    # Two codebooks with ranges 10 and 100: "maximum entry in any table at most 255"
    T = np.concatenate([_table([3, 13]), _table([-50, 50])], axis=0)
    luts, scale, offset, l, delta = oracle.quantize_luts(T)
    assert l[0] == 1 and luts.max() == 200 and luts[0].max() == 20
    assert delta[:, 0].tolist() == [3, -50] and offset[0] == -47.0


def test_quantize_degenerate_column():
    T = np.full((2, 16, 1), 4.5)
    luts, scale, offset, l, _ = oracle.quantize_luts(T)
    assert (luts == 0).all() and scale[0] == 1.0 and l[0] == 0 and offset[0] == 9.0


def test_quantize_invariants_and_error_bound():
    rng = np.random.default_rng(8)
    Cc, M, N = 5, 7, 300
    T = rng.standard_normal((Cc, 16, M)) * rng.uniform(0.01, 50, size=(1, 1, M))
    luts, scale, offset, l, delta = oracle.quantize_luts(T)
    # every table's minimum maps to 0, the column maximum lands in (127.5, 255]
    assert (luts.min(axis=1) == 0).all()
    colmax = luts.reshape(Cc * 16, M).max(axis=0)
    assert ((colmax > 127) & (colmax <= 255)).all()
    # scale is an exact power of two
    mant, _ = np.frexp(scale)
    assert (mant == 0.5).all()
    np.testing.assert_allclose(offset, delta.sum(axis=0).astype(np.float32), rtol=0, atol=0)
    # half a level of rounding error per codebook, errors add over the C codebooks
    # (proof of Lemma F.5): |alpha f + beta - sum_c T_c[code_c]| <= C alpha / 2
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    packed = oracle.pack(codes)
    out, acc16, ov = oracle.scan(packed, Cc, luts, scale, offset)
    exact = oracle.scan_f64(packed, Cc, T)
    slack = 4 * np.finfo(np.float32).eps * (np.abs(exact) + np.abs(offset) + acc16 * scale)
    assert ov == 0
    assert (np.abs(out - exact) <= Cc * scale / 2 + slack).all()
    # and the bound is not vacuous: the error does reach a good part of it
    assert (np.abs(out - exact) / (Cc * scale / 2)).max() > 0.3


def test_pooled_quantization_of_appendix_a():
    # hand example, 2 codebooks x 2 columns (entries beyond the listed ones repeat the first):
    # codebook 0: column 0 {1, 3}, column 1 {2, 11}  -> delta_0 = 1, range 10
    # codebook 1: column 0 {-4, 0}, column 1 {-2, 60} -> delta_1 = -4, range 64
    T = np.zeros((2, 16, 2))
    T[0, :, 0] = 1; T[0, 1, 0] = 3
    T[0, :, 1] = 2; T[0, 1, 1] = 11
    T[1, :, 0] = -4; T[1, 1, 0] = 0
    T[1, :, 1] = -2; T[1, 1, 1] = 60
    luts, scale, offset, l, delta = oracle.quantize_luts_pooled(T)
    assert delta.tolist() == [1.0, -4.0] and l == 1            # 64 * 2 = 128 <= 255 < 256
    assert (scale == 0.5).all() and (offset == -3.0).all()
    assert luts[0, :2, 0].tolist() == [0, 4] and luts[0, :2, 1].tolist() == [2, 20]
    assert luts[1, :2, 0].tolist() == [0, 8] and luts[1, :2, 1].tolist() == [4, 128]
    # one column: pooled and per-column quantisation coincide
    rng = np.random.default_rng(21)
    T1 = rng.standard_normal((4, 16, 1)) * 7
    a = oracle.quantize_luts_pooled(T1)
    b = oracle.quantize_luts(T1)
    assert (a[0] == b[0]).all() and a[1][0] == b[1][0] and a[2][0] == b[2][0]
    # invariants and the half-level error bound with one alpha for all columns
    Cc, M, N = 6, 9, 200
    T = rng.standard_normal((Cc, 16, M)) * rng.uniform(0.1, 20, size=(1, 1, M))
    luts, scale, offset, l, delta = oracle.quantize_luts_pooled(T)
    assert (luts.reshape(Cc, -1).min(axis=1) == 0).all() and 127 < luts.max() <= 255
    assert len(set(scale.tolist())) == 1 and len(set(offset.tolist())) == 1
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    packed = oracle.pack(codes)
    out, acc16, ov = oracle.scan(packed, Cc, luts, scale, offset)
    exact = oracle.scan_f64(packed, Cc, T)
    slack = 4 * np.finfo(np.float32).eps * (np.abs(exact) + np.abs(offset) + acc16 * scale)
    assert (np.abs(out - exact) <= Cc * scale / 2 + slack).all()


# ---------------------------------------------------------------------------
# aggregation f (Section 4.4) and alpha f + beta (Section 1.1)
# ---------------------------------------------------------------------------

def test_scan_equals_integer_matmul_with_one_hot_codes():
    rng = np.random.default_rng(9)
    N, Cc, M = 120, 7, 11           # odd C: last high nibble unused
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    luts = rng.integers(0, 256, size=(Cc, 16, M)).astype(np.uint8)
    scale = (2.0 ** rng.integers(-9, 4, size=M)).astype(np.float32)
    offset = rng.standard_normal(M).astype(np.float32) * 10
    out, acc16, ov, acc32 = oracle.scan(oracle.pack(codes), Cc, luts, scale, offset, want_acc32=True)
    G = _one_hot_rows(codes).astype(np.int64)
    ref = G @ luts.reshape(Cc * 16, M).astype(np.int64)
    assert ov == 0 and (acc32 == ref).all() and (acc16 == ref).all()
    # alpha f + beta with one rounding: compare against exact rational arithmetic
    for n in range(0, N, 17):
        for m in range(M):
            exact = Fraction(int(ref[n, m])) * Fraction(float(scale[m])) + Fraction(float(offset[m]))
            lo, hi = np.nextafter(out[n, m], -np.inf), np.nextafter(out[n, m], np.inf)
            assert abs(Fraction(float(out[n, m])) - exact) <= min(
                abs(Fraction(float(lo)) - exact), abs(Fraction(float(hi)) - exact))
    # rows are independent (Appendix E.2): permuting rows permutes the output
    perm = rng.permutation(N)
    out_p, acc_p, _ = oracle.scan(oracle.pack(codes[perm]), Cc, luts, scale, offset)
    assert (out_p == out[perm]).all() and (acc_p == acc16[perm]).all()


# ---------------------------------------------------------------------------
# aggregation by pairwise averages (Section 4.4; Appendix D)
# ---------------------------------------------------------------------------

def _identity_tables(values):
    """Tables in which code k of codebook c selects values[c][k] (one column)."""
    v = np.asarray(values, dtype=np.uint8)
    return v.reshape(v.shape[0], 16, 1)


def test_averaged_scan_pair_rule_and_constant_blocks():
    one = np.ones(1, np.float32); zero = np.zeros(1, np.float32)
    # U = 2, C = 2: the estimate is 2 floor((a + b + 1) / 2) - 2 * 1 / 4 (Definition D.2, Theorem D.1)
    vals = np.zeros((2, 16), dtype=np.uint8)
    vals[0] = np.arange(16) * 17            # 0, 17, ..., 255
    vals[1] = 255 - np.arange(16) * 16      # 255, 239, ..., 15
    luts = _identity_tables(vals)
    codes = np.array([[i, j] for i in range(16) for j in range(16)], dtype=np.uint8)
    out, usum = oracle.scan_averaged(oracle.pack(codes), 2, luts, one, zero, U=2)
    a = vals[0][codes[:, 0]].astype(int); b = vals[1][codes[:, 1]].astype(int)
    assert (usum[:, 0] == 2 * ((a + b + 1) // 2)).all()
    assert (out[:, 0] == 2 * ((a + b + 1) // 2) - 0.5).all()
    # equal entries in a block: every average is that entry, the estimate is the exact sum minus C log2(U) / 4
    Cc = 32
    luts = np.zeros((Cc, 16, 3), dtype=np.uint8)
    luts[:16] = 100; luts[16:] = 7
    codes = np.random.default_rng(30).integers(0, 16, size=(50, Cc)).astype(np.uint8)
    out, usum = oracle.scan_averaged(oracle.pack(codes), Cc, luts, np.ones(3, np.float32), np.zeros(3, np.float32))
    assert (usum == 16 * 107).all() and (out == 16 * 107 - Cc).all()
    with pytest.raises(ValueError):
        oracle.scan_averaged(oracle.pack(codes[:, :24]), 24, luts[:24], np.ones(3, np.float32), np.zeros(3, np.float32))


def test_averaged_scan_bias_and_range():
    # Lemma D.1 over all 65536 byte pairs: E[2 mu(a, b) - (a + b)] = 1/2 exactly.
    vals = np.zeros((2, 16), dtype=np.uint8)
    rng = np.random.default_rng(31)
    codes = np.array([[i, j] for i in range(16) for j in range(16)], dtype=np.uint8)
    packed2 = oracle.pack(codes)
    acc = []
    for ta in range(16):
        for tb in range(16):
            vals[0] = np.arange(16) + 16 * ta
            vals[1] = np.arange(16) + 16 * tb
            _, usum = oracle.scan_averaged(packed2, 2, _identity_tables(vals), np.ones(1, np.float32),
                                           np.zeros(1, np.float32), U=2)
            a = vals[0][codes[:, 0]].astype(int); b = vals[1][codes[:, 1]].astype(int)
            acc.append(usum[:, 0].astype(int) - (a + b))
    d = np.concatenate(acc)
    assert d.size == 65536 and set(d.tolist()) == {0, 1} and d.mean() == 0.5
    # Theorem D.1, checked the way the paper did (uniform integers 0..255): the excess of
    # U sum(block averages) over the exact sum has mean C log2(U) / 4 and lies in [0, C log2(U) / 2].
    Cc, M, N = 64, 8, 4000
    luts = rng.integers(0, 256, size=(Cc, 16, M)).astype(np.uint8)
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    packed = oracle.pack(codes)
    out, usum = oracle.scan_averaged(packed, Cc, luts, np.ones(M, np.float32), np.zeros(M, np.float32))
    _, _, _, exact = oracle.scan(packed, Cc, luts, np.ones(M, np.float32), np.zeros(M, np.float32), want_acc32=True)
    excess = usum.astype(np.int64) - exact.astype(np.int64)
    assert excess.min() >= 0 and excess.max() <= Cc * 4 // 2
    assert abs(excess.mean() - Cc * 4 / 4) < 0.2            # 64 +- a few standard errors
    assert abs((out - exact).mean()) < 0.2                  # debiased
    # pairs of odd sum round up: a sum of evens is reproduced exactly
    luts_even = luts & 0xF0
    _, usum_e = oracle.scan_averaged(packed, Cc, luts_even, np.ones(M, np.float32), np.zeros(M, np.float32))
    _, _, _, exact_e = oracle.scan(packed, Cc, luts_even, np.ones(M, np.float32), np.zeros(M, np.float32), want_acc32=True)
    assert (usum_e == exact_e).all()


def test_averaged_scan_block_order_by_brute_force():
    """Definition D.2 halves a block recursively; written bottom-up that is: average neighbours
    (0,1), (2,3), ..., then neighbours of the results, four times for U = 16.  Blocks are runs of
    16 consecutive codebooks.  Tiny case, plain Python integers."""
    rng = np.random.default_rng(32)
    Cc, M, N = 32, 2, 40
    luts = rng.integers(0, 256, size=(Cc, 16, M)).astype(np.uint8)
    codes = rng.integers(0, 16, size=(N, Cc)).astype(np.uint8)
    _, usum = oracle.scan_averaged(oracle.pack(codes), Cc, luts, np.ones(M, np.float32), np.zeros(M, np.float32))
    for n in range(N):
        for m in range(M):
            total = 0
            for first in range(0, Cc, 16):
                level = [int(luts[c, codes[n, c], m]) for c in range(first, first + 16)]
                while len(level) > 1:
                    level = [(level[i] + level[i + 1] + 1) // 2 for i in range(0, len(level), 2)]
                total += level[0]
            assert usum[n, m] == 16 * total
    # the order matters (so the check above can fail): pairing codebook c with c + 8 instead of its
    # neighbour changes some results
    perm = np.arange(Cc).reshape(2, 2, 8).transpose(0, 2, 1).reshape(Cc)      # 0, 8, 1, 9, ...
    _, usum_p = oracle.scan_averaged(oracle.pack(codes[:, perm]), Cc, luts[perm], np.ones(M, np.float32),
                                     np.zeros(M, np.float32))
    assert (usum_p != usum).any()


def test_scan_reports_accumulators_beyond_16_bits():
    Cc = 258                        # 258 * 255 = 65790 > 65535
    codes = np.zeros((1, Cc), dtype=np.uint8)
    luts = np.full((Cc, 16, 1), 255, dtype=np.uint8)
    _, _, ov, acc32 = oracle.scan(oracle.pack(codes), Cc, luts, np.ones(1, np.float32),
                                  np.zeros(1, np.float32), want_acc32=True)
    assert ov == 1 and acc32[0, 0] == 65790


def test_encode_scan_is_encode_then_scan():
    rng = np.random.default_rng(10)
    N, D, Cc, M = 90, 10, 4, 6
    A = rng.standard_normal((N, D)).astype(np.float32)
    sd = rng.integers(0, D, size=(Cc, 4)).astype(np.int32)
    th = rng.standard_normal((Cc, 16)).astype(np.float32) * 0.5
    luts = rng.integers(0, 256, size=(Cc, 16, M)).astype(np.uint8)
    scale = np.full(M, 0.25, np.float32); offset = rng.standard_normal(M).astype(np.float32)
    out, acc, packed = oracle.encode_scan(A, sd, th, luts, scale, offset)
    p2 = oracle.pack(oracle.encode(A, sd, th))
    out2, acc2, _ = oracle.scan(p2, Cc, luts, scale, offset)
    assert (packed == p2).all() and (out == out2).all() and (acc == acc2).all()
    # strided rows (lda > D) give the same result
    Abig = np.zeros((N, D + 3), dtype=np.float32); Abig[:, :D] = A
    out3, _, _ = oracle.encode_scan(Abig[:, :D], sd, th, luts, scale, offset)
    assert (out3 == out).all()


# ---------------------------------------------------------------------------
# exact product and NMSE (Section 5.5)
# ---------------------------------------------------------------------------

def test_matmul_and_nmse():
    rng = np.random.default_rng(11)
    A = rng.standard_normal((40, 9)).astype(np.float32)
    B = rng.standard_normal((9, 4)).astype(np.float32)
    Y = oracle.matmul_f64(A, B)
    np.testing.assert_allclose(Y, A.astype(np.float64) @ B.astype(np.float64), rtol=1e-13, atol=1e-13)
    assert oracle.nmse(np.zeros((40, 4), np.float32), Y) == 1.0      # always predicting 0
    Y32 = Y.astype(np.float32)
    assert oracle.nmse(Y32, Y32.astype(np.float64)) == 0.0           # perfect
    assert abs(oracle.nmse((2 * Y).astype(np.float32), Y) - 1.0) < 1e-6


def test_exact_recovery_when_prototypes_reproduce_the_data():
    # Every subvector takes one of 16 values that one coordinate separates, and the
    # prototypes are the bucket means: the reconstruction equals A, so the exact-
    # table output equals A B and the 8-bit output is within C alpha / 2 of it.
    rng = np.random.default_rng(12)
    Cc, w, N, M = 3, 4, 400, 5
    D = Cc * w
    atoms = rng.standard_normal((Cc, 16, w)).astype(np.float32)
    atoms[:, :, 0] = np.arange(16, dtype=np.float32)[None, :] * 3 + rng.uniform(0, 1, (Cc, 16)).astype(np.float32)
    pick = rng.integers(0, 16, size=(N, Cc))
    pick[:16] = np.arange(16)[:, None]            # every atom occurs
    A = np.concatenate([atoms[c, pick[:, c]] for c in range(Cc)], axis=1)
    atoms[:, :, 1:] *= 1e-3                       # coordinate 0 carries the variance
    A = np.ascontiguousarray(np.concatenate([atoms[c, pick[:, c]] for c in range(Cc)], axis=1))
    subspaces = [(c * w, (c + 1) * w) for c in range(Cc)]
    split_dims, thresholds, train_codes, _ = oracle.learn_trees(A, subspaces)
    prototypes = oracle.bucket_means(train_codes, A, subspaces).astype(np.float32)
    B = rng.standard_normal((D, M)).astype(np.float32)
    codes = oracle.encode(A, split_dims, thresholds)
    assert (codes == train_codes).all()
    assert all(len(set(codes[:, c].tolist())) == 16 for c in range(Cc))
    T = oracle.build_luts_f64(prototypes, B)
    Y = oracle.matmul_f64(A, B)
    exact_tables = oracle.scan_f64(oracle.pack(codes), Cc, T)
    np.testing.assert_allclose(exact_tables, Y, rtol=1e-6, atol=1e-6)
    luts, scale, offset, _, _ = oracle.quantize_luts(T)
    out, _, _ = oracle.scan(oracle.pack(codes), Cc, luts, scale, offset)
    assert (np.abs(out - Y) <= Cc * scale / 2 + 1e-5).all()
