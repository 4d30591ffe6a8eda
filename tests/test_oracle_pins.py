"""Pins for the CPU oracle: each test checks it against something other than itself --
values fixed by the paper's format rules, exact rational arithmetic, closed forms,
invariants and library routines.  No GPU."""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "packed_words.txt")
BITS = (2, 3, 4)


def _golden_cases():
    cases = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, codes, words = [p.strip() for p in line.split("|")]
            cases.append((int(b), [int(c) for c in codes.split()], [int(w, 16) for w in words.split()]))
    return cases


# ------------------------------------------------------------------ packing (Section 3, Alg. 2)

@pytest.mark.parametrize("bits,codes,words", _golden_cases())
def test_pack_matches_paper_word_format(oracle, bits, codes, words):
    q = np.array([codes], np.uint8)                    # one output, K = len(codes)
    P = oracle.pack_codes(q, bits)
    assert P.shape == (len(words), 1)
    assert [int(w) for w in P[:, 0]] == words
    assert oracle.unpack_codes(P, len(codes), bits).tolist() == [codes]


@pytest.mark.parametrize("bits", BITS)
def test_pack_equals_bitstream_integer(oracle, bits):
    # Alg. 2 read backwards: the packed words of one output are the little-endian digits
    # (base 2^32) of sum_k q_k * 2^(b k).  Computed here with Python integers.
    rng = np.random.default_rng(7 + bits)
    N, K = 5, 96
    q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
    P = oracle.pack_codes(q, bits)
    for n in range(N):
        v = sum(int(c) << (bits * k) for k, c in enumerate(q[n]))
        for w in range(P.shape[0]):
            assert int(P[w, n]) == (v >> (32 * w)) & 0xFFFFFFFF


@pytest.mark.parametrize("bits", BITS)
def test_pack_sizes_and_storage_formula(oracle, bits):
    # Section 3: 32/b codes per word (3-bit: 32 codes per 3 words); storage of a matrix with
    # one group per output is b*K*N + 32*N + b*N bits.
    N, K = 12, 64
    q = np.zeros((N, K), np.uint8)
    P = oracle.pack_codes(q, bits)
    assert P.shape == (K * bits // 32, N)
    assert oracle.storage_bits(N, K, bits, K) == bits * K * N + 32 * N + bits * N
    G = 16
    assert oracle.storage_bits(N, K, bits, G) == bits * K * N + (32 + bits) * N * (K // G)


def test_pack_orientation_is_input_dim_major(oracle):
    # Section 3: entry (i, j) of the 4-bit packed matrix holds rows 8i..8i+7 of column j of
    # the uncompressed matrix (the paper's rows are inputs k, its columns outputs n).
    N, K = 3, 32
    for n in range(N):
        for k in range(K):
            q = np.zeros((N, K), np.uint8)
            q[n, k] = 9
            P = oracle.pack_codes(q, 4)
            nz = np.argwhere(P != 0)
            assert nz.tolist() == [[k // 8, n]]
            assert int(P[k // 8, n]) == 9 << (4 * (k % 8))


@pytest.mark.parametrize("bits", BITS)
def test_pack_unpack_identity(oracle, bits):
    rng = np.random.default_rng(bits)
    for N, K in ((1, 32), (7, 160), (64, 512)):
        q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
        assert np.array_equal(oracle.unpack_codes(oracle.pack_codes(q, bits), K, bits), q)
    # zero-points: stream length need not fill a word; padding bits are zero
    for N, G in ((3, 1), (5, 7), (4, 33)):
        z = rng.integers(0, 1 << bits, (N, G), dtype=np.uint8)
        Zp = oracle.pack_zeros(z, bits)
        assert Zp.shape == ((G * bits + 31) // 32, N)
        assert np.array_equal(oracle.unpack_zeros(Zp, G, bits), z)
        total = Zp.shape[0] * 32
        for n in range(N):
            v = sum(int(w) << (32 * i) for i, w in enumerate(Zp[:, n]))
            assert v >> (G * bits) == 0 and total >= G * bits


def test_pack_rejects_out_of_range_code(oracle):
    q = np.zeros((1, 32), np.uint8)
    q[0, 3] = 4
    with pytest.raises(ValueError):
        oracle.pack_codes(q, 2)


def test_scales_canonical_is_transpose(oracle):
    s = np.arange(12, dtype=np.float32).reshape(3, 4)
    assert np.array_equal(oracle.transpose_scales(s), s.T)


# ------------------------------------------------------------------ quantizer (Section 2)

def _frac(a):
    return Fraction(float(a))


@pytest.mark.parametrize("bits", BITS)
def test_codes_in_range_and_error_bound(oracle, bits):
    # Q maps into [0, 2^b); rounding to nearest leaves |D(Q(w)) - w| <= s/2 (up to fp32
    # rounding of the quotient), for every weight, because the range contains 0 and so the
    # grid covers [lo, hi] up to half a step at either end.
    rng = np.random.default_rng(11 * bits)
    W = (rng.standard_normal((16, 256)) * 0.02).astype(np.float32)
    W[rng.random(W.shape) < 0.01] *= 20
    G = 32
    q, s, z = oracle.quantize(W, bits, G)
    assert q.min() >= 0 and q.max() <= (1 << bits) - 1
    assert z.min() >= 0 and z.max() <= (1 << bits) - 1
    What = oracle.dequantize(q, s, z, G)
    S = np.repeat(s.astype(np.float64), G, axis=1)
    assert np.all(np.abs(What - W.astype(np.float64)) <= S / 2 * (1 + 2.0 ** -20))


@pytest.mark.parametrize("bits", BITS)
def test_scale_is_correctly_rounded_range_over_levels(oracle, bits):
    # s = (hi - lo) / (2^b - 1) with lo <= 0 <= hi: checked in exact rationals -- s must be
    # the float32 nearest to fl32(hi - lo) / (2^b - 1).
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((8, 64)) * 0.02).astype(np.float32)
    G = 16
    _, s, _ = oracle.quantize(W, bits, G)
    for n in range(W.shape[0]):
        for g in range(W.shape[1] // G):
            w = W[n, g * G:(g + 1) * G]
            lo, hi = min(np.float32(0), w.min()), max(np.float32(0), w.max())
            r = np.float32(hi) - np.float32(lo)           # one fp32 subtraction
            exact = _frac(r) / ((1 << bits) - 1)
            got = s[n, g]
            err = abs(_frac(got) - exact)
            up, dn = np.nextafter(got, np.float32(np.inf)), np.nextafter(got, np.float32(-np.inf))
            assert err <= abs(_frac(up) - exact) and err <= abs(_frac(dn) - exact)


@pytest.mark.parametrize("bits", BITS)
def test_codes_are_nearest_grid_points_bruteforce(oracle, bits):
    # RTN means: q is the code c in [0, 2^b - 1] whose grid point s*(c - z) is nearest to w;
    # z is the code nearest to -lo/s.  Brute force over all codes in exact rationals; inputs
    # whose two nearest candidates are closer than 2^-20 of a step are skipped (fp32 rounding
    # of the quotient may legitimately decide those either way).
    rng = np.random.default_rng(100 + bits)
    W = (rng.standard_normal((6, 48)) * 0.02).astype(np.float32)
    G = 16
    qmax = (1 << bits) - 1
    q, s, z = oracle.quantize(W, bits, G)
    checked = 0
    for n in range(W.shape[0]):
        for g in range(W.shape[1] // G):
            sf = _frac(s[n, g])
            w = W[n, g * G:(g + 1) * G]
            lo = min(Fraction(0), min(_frac(v) for v in w))
            dz = sorted((abs(sf * c + lo), c) for c in range(qmax + 1))
            if dz[1][0] - dz[0][0] > sf / 2 ** 20:
                assert int(z[n, g]) == dz[0][1]
            zz = int(z[n, g])
            for k, v in enumerate(w):
                d = sorted((abs(sf * (c - zz) - _frac(v)), c) for c in range(qmax + 1))
                if d[1][0] - d[0][0] > sf / 2 ** 20:
                    assert int(q[n, g * G + k]) == d[0][1]
                    checked += 1
    assert checked > 250


@pytest.mark.parametrize("bits", BITS)
def test_matches_paper_Q_when_minimum_is_on_the_grid(oracle, bits):
    # Section 2: Q(x,b) = rnd((x - min)/(max - min) * (2^b - 1)).  With min <= 0 <= max and
    # -min an exact multiple of the step, the integer-zero form q = rnd(w/s) + z coincides
    # with it.  Step 2^-6 and integer multiples keep every quantity exact.
    qmax = (1 << bits) - 1
    step = Fraction(1, 64)
    rng = np.random.default_rng(3)
    for zero in range(qmax + 1):
        lo, hi = -zero * step, (qmax - zero) * step
        G = 32
        vals = [lo, hi] + [lo + Fraction(int(t), 4096) * (hi - lo) for t in rng.integers(0, 4097, G - 2)]
        W = np.array([[float(v) for v in vals]], np.float32)
        assert all(_frac(a) == b for a, b in zip(W[0], vals))
        q, s, z = oracle.quantize(W, bits, G)
        assert _frac(s[0, 0]) == step and int(z[0, 0]) == zero
        for k, v in enumerate(vals):
            t = (v - lo) / (hi - lo) * qmax                      # the paper's argument of rnd
            if t.denominator == 2:                                # exact tie: skip
                continue
            assert int(q[0, k]) == round(t)


@pytest.mark.parametrize("bits", BITS)
def test_endpoints_map_to_extreme_codes(oracle, bits):
    # Q maps min -> 0 and max -> 2^b - 1 (Section 2) whenever min < 0 < max.
    rng = np.random.default_rng(17)
    W = (rng.standard_normal((32, 64)) * 0.02).astype(np.float32)
    G = 32
    q, s, z = oracle.quantize(W, bits, G)
    qmax = (1 << bits) - 1
    hits_hi = 0
    for n in range(W.shape[0]):
        for g in range(2):
            w = W[n, g * G:(g + 1) * G]
            qq = q[n, g * G:(g + 1) * G]
            assert qq[np.argmin(w)] == 0
            assert qq[np.argmax(w)] in (qmax, qmax - 1)       # qmax-1 only at an exact .5 tie
            hits_hi += qq[np.argmax(w)] == qmax
    assert hits_hi >= 60


@pytest.mark.parametrize("bits", BITS)
def test_grid_exact_weights_round_trip_exactly(oracle, bits):
    # Weights that already lie on a grid s0*(q0 - z0), s0 a power of two, using both extreme
    # codes: the quantizer must return exactly (q0, s0, z0) and D must return W exactly.
    qmax = (1 << bits) - 1
    rng = np.random.default_rng(23)
    G, N, K = 32, 8, 128
    q0 = rng.integers(0, qmax + 1, (N, K), dtype=np.uint8)
    z0 = rng.integers(0, qmax + 1, (N, K // G), dtype=np.uint8)
    s0 = (2.0 ** rng.integers(-9, -3, (N, K // G))).astype(np.float32)
    q0[:, 0::G] = 0
    q0[:, 1::G] = qmax
    W = (np.repeat(s0, G, 1).astype(np.float64) * (q0.astype(np.int32) - np.repeat(z0, G, 1).astype(np.int32))).astype(np.float32)
    q, s, z = oracle.quantize(W, bits, G)
    assert np.array_equal(s, s0) and np.array_equal(z, z0) and np.array_equal(q, q0)
    assert np.array_equal(oracle.dequantize(q, s, z, G), W.astype(np.float64))


def test_ties_round_half_to_even(oracle):
    # s = 1 exactly (range 15 at 4 bits, 0 included): w = k + 0.5 must go to the even code.
    W = np.array([[0.0, 15.0, 0.5, 1.5, 2.5, 3.5, 6.5, 13.5] + [0.0] * 8], np.float32)
    q, s, z = oracle.quantize(W, 4, 16)
    assert s[0, 0] == 1.0 and z[0, 0] == 0
    assert q[0, :8].tolist() == [0, 15, 0, 2, 2, 4, 6, 14]
    # with an odd zero-point the tie is decided on w/s before the integer zero is added:
    # rnd(0.5) + 1 = 1 and rnd(1.5) + 1 = 3 (not rnd(0.5 + 1) = 2, rnd(1.5 + 1) = 2).
    W = np.array([[-1.0, 14.0, 0.5, 1.5, 2.5, -0.5] + [0.0] * 10], np.float32)
    q, s, z = oracle.quantize(W, 4, 16)
    assert s[0, 0] == 1.0 and z[0, 0] == 1
    assert q[0, :6].tolist() == [0, 15, 1, 3, 3, 1]


@pytest.mark.parametrize("bits", BITS)
def test_one_sided_and_degenerate_groups(oracle, bits):
    qmax = (1 << bits) - 1
    G = 16
    pos = np.linspace(0.25, 1.0, G, dtype=np.float32)          # all positive: lo = 0 -> z = 0
    neg = -pos                                                 # all negative: hi = 0 -> z = qmax
    zero = np.zeros(G, np.float32)                             # range 0 -> s = 1, z = 0, q = 0
    W = np.stack([pos, neg, zero])
    q, s, z = oracle.quantize(W, bits, G)
    assert z[:, 0].tolist() == [0, qmax, 0]
    assert s[2, 0] == 1.0 and not q[2].any()
    assert _frac(s[0, 0]) == _frac(np.float32(1.0) / np.float32(qmax))
    assert q[0].max() == qmax and q[1].min() == 0
    What = oracle.dequantize(q, s, z, G)
    assert np.all(np.abs(What - W) <= s.astype(np.float64) / 2 * (1 + 2.0 ** -20))


def test_groups_run_along_the_input_dimension(oracle):
    # A single large entry must change the scale of exactly its own (n, k // G) group.
    N, K, G = 4, 64, 16
    W = np.full((N, K), 0.01, np.float32)
    _, s0, _ = oracle.quantize(W, 4, G)
    W[2, 37] = 5.0
    _, s1, _ = oracle.quantize(W, 4, G)
    assert np.argwhere(s0 != s1).tolist() == [[2, 37 // G]]


# ------------------------------------------------------------------ products (eq. (1), (2), Alg. 1)

def _case(rng, N, K, G, bits):
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    x = rng.standard_normal(K).astype(np.float32)
    return W, x


@pytest.mark.parametrize("bits", BITS)
def test_matvec_equals_numpy_on_dequantized_matrix(oracle, bits):
    rng = np.random.default_rng(31 + bits)
    N, K, G = 37, 96, 32                                       # non-square: catches a transpose
    W, x = _case(rng, N, K, G, bits)
    q, s, z = oracle.quantize(W, bits, G)
    What = oracle.dequantize(q, s, z, G)
    ref = What @ x.astype(np.float64)
    y = oracle.matvec(q, s, z, G, x)
    assert np.allclose(y, ref, rtol=0, atol=1e-13 * np.abs(What).sum(1).max() * np.abs(x).max())
    # and the dequantized matrix itself against the definition s*(q - z), by numpy
    ref_W = np.repeat(s, G, 1).astype(np.float64) * (q.astype(np.float64) - np.repeat(z, G, 1))
    assert np.array_equal(What, ref_W)


@pytest.mark.parametrize("bits", BITS)
def test_matvec_unit_scale_zero_offset_is_integer_matmul(oracle, bits):
    rng = np.random.default_rng(41)
    N, K, G = 19, 128, 32
    q = rng.integers(0, 1 << bits, (N, K), dtype=np.uint8)
    s = np.ones((N, K // G), np.float32)
    z = np.zeros((N, K // G), np.uint8)
    x = rng.integers(-50, 51, K).astype(np.float32)
    y = oracle.matvec(q, s, z, G, x)
    exact = q.astype(np.int64) @ x.astype(np.int64)
    assert np.array_equal(y, exact.astype(np.float64))
    assert np.array_equal(oracle.matvec_factored(q, s, z, G, x), exact.astype(np.float64))


@pytest.mark.parametrize("bits", BITS)
def test_matvec_zero_input_gives_zero(oracle, bits):
    rng = np.random.default_rng(43)
    W, _ = _case(rng, 9, 64, 16, bits)
    q, s, z = oracle.quantize(W, bits, 16)
    assert not oracle.matvec(q, s, z, 16, np.zeros(64, np.float32)).any()


@pytest.mark.parametrize("bits", BITS)
def test_factored_form_equals_direct_form(oracle, bits):
    # eq. (2) (with the scale kept on the zero term) against the left-hand side; also eq. (1)
    # when there is a single group.
    rng = np.random.default_rng(47)
    for N, K, G in ((11, 256, 32), (5, 128, 128)):
        W, x = _case(rng, N, K, G, bits)
        q, s, z = oracle.quantize(W, bits, G)
        a = oracle.matvec(q, s, z, G, x)
        b = oracle.matvec_factored(q, s, z, G, x)
        scale = (np.abs(oracle.dequantize(q, s, z, G)) @ np.abs(x.astype(np.float64))).max()
        assert np.max(np.abs(a - b)) <= 1e-12 * scale * (1 << bits)
        if G == K:   # eq. (1): s * (<x, q> - z * <x, 1>), evaluated exactly with integers*floats in numpy
            xd = x.astype(np.float64)
            ref = s[:, 0].astype(np.float64) * (q.astype(np.float64) @ xd - z[:, 0] * xd.sum())
            assert np.max(np.abs(a - ref)) <= 1e-12 * scale * (1 << bits)


@pytest.mark.parametrize("bits", BITS)
def test_matvec_linearity_and_group_permutation(oracle, bits):
    rng = np.random.default_rng(53)
    N, K, G = 13, 192, 32
    W, x = _case(rng, N, K, G, bits)
    x2 = rng.standard_normal(K).astype(np.float32)
    q, s, z = oracle.quantize(W, bits, G)
    y1, y2 = oracle.matvec(q, s, z, G, x), oracle.matvec(q, s, z, G, x2)
    # exact powers of two keep x representable: y(2x) = 2 y(x) exactly
    assert np.array_equal(oracle.matvec(q, s, z, G, x * 2), 2 * y1)
    xs = (x.astype(np.float64) + x2.astype(np.float64)).astype(np.float32)
    if np.array_equal(xs.astype(np.float64), x.astype(np.float64) + x2.astype(np.float64)):
        assert np.allclose(oracle.matvec(q, s, z, G, xs), y1 + y2, rtol=1e-12)
    # permuting whole groups of k together with x leaves y unchanged (up to summation order)
    perm = rng.permutation(K // G)
    idx = (perm[:, None] * G + np.arange(G)[None, :]).ravel()
    yp = oracle.matvec(q[:, idx], s[:, perm], z[:, perm], G, x[idx])
    assert np.allclose(yp, y1, rtol=0, atol=1e-12)


@pytest.mark.parametrize("bits", BITS)
def test_packed_matvec_equals_unpacked(oracle, bits):
    rng = np.random.default_rng(59)
    N, K, G = 21, 160, 32
    W, x = _case(rng, N, K, G, bits)
    q, s, z = oracle.quantize(W, bits, G)
    y = oracle.matvec(q, s, z, G, x)
    yp = oracle.matvec_packed(oracle.pack_codes(q, bits), oracle.transpose_scales(s),
                              oracle.pack_zeros(z, bits), K, bits, G, x)
    assert np.array_equal(y, yp)


@pytest.mark.parametrize("bits", BITS)
def test_matmul_small_rows_equal_matvec_and_numpy(oracle, bits):
    rng = np.random.default_rng(61)
    N, K, G, M = 17, 96, 32, 5
    W, _ = _case(rng, N, K, G, bits)
    X = rng.standard_normal((M, K)).astype(np.float32)
    q, s, z = oracle.quantize(W, bits, G)
    Y = oracle.matmul_small(q, s, z, G, X)
    assert Y.shape == (M, N)
    for m in range(M):
        assert np.array_equal(Y[m], oracle.matvec(q, s, z, G, X[m]))
    ref = X.astype(np.float64) @ oracle.dequantize(q, s, z, G).T
    assert np.allclose(Y, ref, rtol=0, atol=1e-12)


def test_row_norms_match_numpy(oracle):
    rng = np.random.default_rng(67)
    W, _ = _case(rng, 9, 64, 16, 4)
    q, s, z = oracle.quantize(W, 4, 16)
    ref = np.linalg.norm(oracle.dequantize(q, s, z, 16), axis=1)
    assert np.allclose(oracle.row_norms(q, s, z, 16), ref, rtol=1e-14)


# ------------------------------------------------------------------ gated combination (silu(g) * u)

def test_swiglu_against_identities(oracle):
    # silu(t) = t * sigmoid(t): checked against the tanh form of the sigmoid, the odd-part identity
    # silu(t) - silu(-t) = t, its values at 0 and far out, and linearity in u
    rng = np.random.default_rng(11)
    g = np.concatenate([rng.standard_normal(200) * 4.0, [0.0, 50.0, -50.0, 1e-9]])
    u = rng.standard_normal(g.size)
    one = np.ones_like(g)
    silu = oracle.swiglu(g, one)
    near = np.abs(g) < 12.0          # further out 1 + tanh cancels; the limits below cover that range
    assert np.allclose(silu[near], (g * 0.5 * (1.0 + np.tanh(0.5 * g)))[near], rtol=1e-9, atol=1e-300)
    assert np.allclose(silu - oracle.swiglu(-g, one), g, rtol=1e-13, atol=1e-15)
    assert silu[200] == 0.0 and abs(silu[201] - 50.0) < 1e-19 * 50 + 1e-15 and abs(silu[202]) < 1e-19
    assert np.allclose(oracle.swiglu(g, u), silu * u, rtol=1e-15)
    assert np.allclose(oracle.swiglu(g, 3.0 * u), 3.0 * oracle.swiglu(g, u), rtol=1e-15)
    # derivative at 0 is 1/2: silu(t) ~ t/2 + t^2/4 for small t
    t = np.array([1e-4])
    assert abs(oracle.swiglu(t, np.ones(1))[0] - (t[0] / 2 + t[0] ** 2 / 4)) < 1e-13

