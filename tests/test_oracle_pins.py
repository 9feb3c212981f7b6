"""Pins for the CPU oracle: each check ties an oracle function to something
that is not the oracle's own formula -- LAPACK's SVD, a closed form, a
brute-force loop, an invariant from the paper, or a value the paper prints.
CPU only."""
import itertools
import os

import numpy as np
import pytest

import workloads as wl
from oracle import signmuon_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
SHAPES = [(8, 8), (12, 5), (5, 12), (32, 17), (17, 32), (1, 9), (9, 1)]


def svd_polar(X):
    """Definition (Polar factor): U V^T from a thin SVD, on the support."""
    U, s, Vt = np.linalg.svd(X, full_matrices=False)
    keep = s > s.max() * 1e-12
    return (U[:, keep]) @ Vt[keep], U, s, Vt


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("shape", SHAPES)
def test_ns_converges_to_svd_polar(shape):
    X, *_ = wl.with_condition(*shape, cond=50.0, seed=1)
    X = 7.3 * X
    Q, *_ = svd_polar(X)
    Y = O.polar_ns(X, steps=60, scale="fro")
    assert np.linalg.norm(Y - Q) <= 1e-9


# ---------------------------------------------------------------- P2
@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("coeffs,K", [((1.5, -0.5, 0.0), 5), ((1.5, -0.5, 0.0), 1),
                                      ((3.4445, -4.7750, 2.0315), 3), ((2.0, -1.5, 0.5), 4)])
def test_ns_matches_per_singular_value_closed_form(shape, coeffs, K):
    """Substituting Y = U S V^T into the iteration: each singular value goes
    through phi(x) = a x + b x^3 + c x^5 K times; U and V do not move."""
    X, *_ = wl.with_condition(*shape, cond=20.0, seed=2)
    X = 0.37 * X
    U, s, Vt = np.linalg.svd(X, full_matrices=False)
    a, b, c = coeffs
    x = s / np.sqrt(np.sum(s * s))            # Frobenius scale
    for _ in range(K):
        x = a * x + b * x ** 3 + c * x ** 5
    expect = (U * x) @ Vt
    for gram in ("short", "paper"):
        Y = O.polar_ns(X, steps=K, coeffs=coeffs, scale="fro", gram=gram)
        assert np.max(np.abs(Y - expect)) <= 1e-10 * max(1.0, np.max(np.abs(expect)))


def test_gram_side_is_immaterial():
    X, *_ = wl.with_condition(6, 40, cond=10.0, seed=3)
    a = O.polar_ns(X, 5, gram="short")
    b = O.polar_ns(X, 5, gram="paper")
    assert np.max(np.abs(a - b)) <= 1e-12
    with pytest.raises(ValueError):
        O.polar_ns(X, 1, gram="other")


# ---------------------------------------------------------------- P3
def test_orthogonal_matrix_is_a_fixed_point():
    g = wl.rng_for(7)
    Q, _ = np.linalg.qr(g.standard_normal((16, 16)))
    for K in (1, 2, 5):
        assert np.max(np.abs(O.polar_ns(Q, K, scale="none") - Q)) <= 1e-13
    # semi-orthogonal (tall and wide), both Gram sides
    Qt, _ = np.linalg.qr(g.standard_normal((20, 6)))
    assert np.max(np.abs(O.polar_ns(Qt, 3, scale="none") - Qt)) <= 1e-13
    assert np.max(np.abs(O.polar_ns(Qt.T, 3, scale="none") - Qt.T)) <= 1e-13
    assert np.linalg.norm(O.polar_ns(Q, 60, scale="fro") - Q) <= 1e-9


# ---------------------------------------------------------------- P4
def test_spectrum_invariants_and_error_recursion():
    X, *_ = wl.with_condition(10, 24, cond=30.0, seed=4)
    prev_sv, prev_E = None, None
    for K in range(0, 9):
        Y = O.polar_ns(X, K, scale="fro")
        sv = np.linalg.svd(Y, compute_uv=False)
        assert sv.max() <= 1.0 + 1e-12 and sv.min() > 0.0          # ||Y_K||_op <= 1
        if prev_sv is not None:
            assert np.all(sv >= prev_sv - 1e-12)                      # non-decreasing
        E = np.linalg.norm(np.eye(10) - Y @ Y.T, 2)                   # short-side Gram
        if prev_E is not None:
            assert E <= prev_E ** 2 + 1e-12                           # ||E_{k+1}|| <= ||E_k||^2
        prev_sv, prev_E = sv, E
    # Theorem (quadratic convergence): ||Y_K - Q||_op <= rho^(2^K)
    Q, *_ = svd_polar(X)
    Y0 = X / np.linalg.norm(X)
    rho = np.linalg.norm(np.eye(10) - Y0 @ Y0.T, 2)
    for K in (2, 5, 8, 12):
        assert np.linalg.norm(O.polar_ns(X, K) - Q, 2) <= rho ** (2 ** K) + 1e-12


def test_rank_deficient_input_stays_on_its_support():
    g = wl.rng_for(8)
    X = g.standard_normal((12, 3)) @ g.standard_normal((3, 9))       # rank 3
    Q, *_ = svd_polar(X)
    Y = O.polar_ns(X, 30)      # zero directions hold only rounding noise, which grows 1.5x a step
    assert np.linalg.norm(Y - Q) <= 1e-8
    assert np.linalg.matrix_rank(Y, tol=1e-6) == 3


# ---------------------------------------------------------------- P5
def test_duality_with_nuclear_norm():
    X, _, sv, _ = wl.with_condition(9, 14, cond=8.0, seed=5)
    Y = O.polar_ns(X, 60)
    assert abs(np.sum(X * Y) - np.sum(sv)) <= 1e-9
    assert abs(np.linalg.norm(Y, 2) - 1.0) <= 1e-9


# ---------------------------------------------------------------- P6
def test_equivariances():
    g = wl.rng_for(9)
    X = g.standard_normal((7, 11))
    Y = O.polar_ns(X, 5)
    assert np.max(np.abs(O.polar_ns(-X, 5) + Y)) <= 1e-13
    assert np.max(np.abs(O.polar_ns(X.T, 5) - Y.T)) <= 1e-13
    assert np.max(np.abs(O.polar_ns(4.5 * X, 5) - Y)) <= 1e-13
    P, R = g.permutation(7), g.permutation(11)
    assert np.max(np.abs(O.polar_ns(X[P][:, R], 5) - Y[P][:, R])) <= 1e-13
    # idealized algorithm: free scaling alpha (scale="none" on X/alpha)
    alpha = 1.3 * np.linalg.norm(X, 2)
    Z = O.polar_ns(X / alpha, 4, scale="none")
    U, s, Vt = np.linalg.svd(X, full_matrices=False)
    x = s / alpha
    for _ in range(4):
        x = 1.5 * x - 0.5 * x ** 3
    assert np.max(np.abs(Z - (U * x) @ Vt)) <= 1e-12


def test_zero_input_gives_zero_without_nan():
    Y = O.polar_ns(np.zeros((4, 6)), 5)
    assert np.all(Y == 0.0)
    Yf = O.polar_ns(np.zeros((4, 6), np.float32), 5, dtype=np.float32)
    assert Yf.dtype == np.float32 and np.all(Yf == 0.0)


def test_eps_floor_on_sigma():
    X = np.full((2, 2), 1e-20)
    Y = O.polar_ns(X, 0, eps=1e-12)
    assert np.allclose(Y, 1e-8, rtol=1e-12)        # divided by eps, not by ||X||_F = 2e-20


# ---------------------------------------------------------------- P7
def test_power_iter():
    g = wl.rng_for(10)
    X = g.standard_normal((13, 21))
    smax = np.linalg.svd(X, compute_uv=False)[0]
    v0 = g.standard_normal(21)
    est = [O.power_iter(X, P, 1e-12, v0) for P in (0, 1, 2, 5, 50, 400)]
    assert all(e <= smax + 1e-12 for e in est)
    assert all(b >= a - 1e-12 for a, b in zip(est, est[1:]))
    assert abs(est[-1] - smax) <= 1e-9
    # P = 0 is ||X v0|| / (||v0|| + eps)
    assert abs(est[0] - np.linalg.norm(X @ v0) / np.linalg.norm(v0)) <= 1e-10
    # rank one: a b^T has norm |a||b| after a single round
    a, b = g.standard_normal(13), g.standard_normal(21)
    assert abs(O.power_iter(np.outer(a, b), 1, 1e-12, v0)
               - np.linalg.norm(a) * np.linalg.norm(b)) <= 1e-9
    # spectral scaling in PolarNS divides by exactly that estimate
    Y = O.polar_ns(X, 0, scale="spectral", power_iters=2, v0=v0)
    assert np.max(np.abs(Y * O.power_iter(X, 2, 1e-12, v0) - X)) <= 1e-12
    with pytest.raises(ValueError):
        O.polar_ns(X, 1, scale="spectral")


def test_fro_scale_value():
    X = np.array([[3.0, 0.0], [0.0, 4.0]])
    assert O.scale_sigma(X, "fro") == 5.0
    assert np.array_equal(O.polar_ns(X, 0, scale="fro"), X / 5.0)


# ---------------------------------------------------------------- P8
@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 8, 12])
def test_vote_exhaustive_against_scalar_definition(M):
    pats = np.array(list(itertools.product([-1, 1], repeat=M)), dtype=np.int8).T   # [M, 2^M]
    d = pats.shape[1]
    expect = []
    for j in range(d):
        s = sum(int(v) for v in pats[:, j])
        expect.append(1 if s >= 0 else -1)                # sign of the sum, ties -> +1
    expect = np.array(expect, dtype=np.int8)
    vote8, tot = O.majority_vote_int8(pats)
    assert np.array_equal(vote8, expect)
    assert np.array_equal(tot, pats.astype(np.int64).sum(0))
    packed = np.stack([O.pack_bits((pats[p] > 0).astype(np.uint8)) for p in range(M)])
    vote1, c = O.majority_vote_bits(packed, M, d)
    assert np.array_equal(vote1, expect)
    assert np.array_equal(2 * c - M, tot)                 # sum = 2c - M


# ---------------------------------------------------------------- P9
def test_vote_symmetries():
    g = wl.rng_for(11)
    for M in (3, 4, 9, 16):
        S = g.choice(np.array([-1, 1], np.int8), size=(M, 1000))
        v, tot = O.majority_vote_int8(S)
        vf, totf = O.majority_vote_int8(-S)
        assert np.array_equal(totf, -tot)
        assert np.array_equal(vf[tot != 0], -v[tot != 0])
        assert np.all(vf[tot == 0] == 1) and np.all(v[tot == 0] == 1)
        assert np.array_equal(O.majority_vote_int8(S[g.permutation(M)])[0], v)
        assert np.array_equal(O.majority_vote_int8(np.concatenate([S, S]))[0], v)
        if M % 2 == 1:
            assert np.all(tot != 0)
    one = g.choice(np.array([-1, 1], np.int8), size=(1, 77))
    assert np.array_equal(O.majority_vote_int8(one)[0], one[0])        # M = 1 is identity
    una = np.tile(one, (5, 1))
    assert np.array_equal(O.majority_vote_int8(una)[0], one[0])        # unanimity


# ---------------------------------------------------------------- P10
@pytest.mark.parametrize("d", [1, 7, 8, 9, 63, 64, 65, 127, 128, 1000])
def test_pack_layout_and_round_trip(d):
    bits = wl.rng_for(12, block=d).integers(0, 2, size=d).astype(np.uint8)
    packed = O.pack_bits(bits)
    assert packed.dtype == np.uint8 and packed.size == 8 * ((d + 63) // 64)
    assert O.packed_bytes(d) == (d + 7) // 8
    for i in range(d):                                   # entry i -> bit i%8 of byte i//8
        assert (packed[i // 8] >> (i % 8)) & 1 == bits[i]
    words = packed.view("<u8")                           # == bit i%64 of LE word i//64
    for i in range(d):
        assert (int(words[i // 64]) >> (i % 64)) & 1 == bits[i]
    tail = np.unpackbits(packed, bitorder="little")[d:]
    assert not tail.any()                                # padding bits are zero
    assert np.array_equal(O.unpack_bits(packed, d), bits)


def test_sign_decision_on_special_values():
    x = wl.special_values_f32()
    expect = np.array([1, 1, 0, 0, 1, 0, 1, 0, 1, 0, 1, 0, 1, 0, 1, 0], np.uint8)
    assert np.array_equal(O.sign_entries(x), expect)
    assert np.array_equal(O.signs_pm1(x), 2 * expect.astype(np.int8) - 1)
    xb = wl.from_bf16_bits(wl.to_bf16_bits(x))           # bf16 rounding takes -1e-45 to -0.0 -> bit 1
    expect_b = expect.copy()
    expect_b[7] = 1
    assert np.array_equal(O.sign_entries(xb), expect_b)
    # the same decision on the raw bit pattern u: (u <= +inf bits) or (u == -0.0 bits)
    u = x.view(np.uint32)
    assert np.array_equal(((u <= 0x7F800000) | (u == 0x80000000)).astype(np.uint8), expect)
    # decoding: 0 -> -1, 1 -> +1
    assert np.array_equal(2 * O.unpack_bits(O.pack_bits(expect), 16).astype(int) - 1,
                          O.signs_pm1(x))


# ---------------------------------------------------------------- P11
def test_payload_sizes_match_papers_worked_example():
    row = [l for l in open(os.path.join(HERE, "golden", "resnet50_payload.txt"))
           if not l.startswith("#")][0].split()
    d, fp32_mb, int8_mb, packed_mib = int(row[0]), float(row[1]), float(row[2]), float(row[3])
    assert abs(4 * d / 1e6 - fp32_mb) < 0.5
    assert abs(d / 1e6 - int8_mb) < 0.05
    assert abs(O.packed_bytes(d) / 2 ** 20 - packed_mib) < 0.05
    assert O.packed_bytes(d) * 32 == 4 * d                # the 32x bandwidth-term cut


# ---------------------------------------------------------------- P12
def test_step_degenerates_to_signsgd():
    g = wl.rng_for(13)
    W = g.standard_normal((6, 10))
    G = g.standard_normal((1, 6, 10))
    out = O.signmuon_step(W, np.zeros_like(G), G, beta=0.0, lr=0.25, ns_steps=0)
    assert np.array_equal(out["W"], W - 0.25 * np.sign(G[0]))
    assert np.array_equal(out["mom"], G)


def test_step_on_all_zero_gradients():
    W = np.ones((4, 16))
    Z = np.zeros((3, 4, 16))
    out = O.signmuon_step(W, Z, Z, beta=0.9, lr=0.5, ns_steps=5)
    assert np.all(out["vote"] == 1) and np.all(out["W"] == 0.5)
    assert not np.isnan(out["U"]).any()


def test_step_composes_the_stages():
    g = wl.rng_for(14)
    M, r, c = 5, 8, 24
    W = g.standard_normal((r, c))
    mom = g.standard_normal((M, r, c))
    G = g.standard_normal((M, r, c))
    for fmt in ("1bit", "int8"):
        out = O.signmuon_step(W, mom, G, beta=0.9, weight_decay=0.1, lr=1e-2, ns_steps=3,
                              sign_fmt=fmt, local_polar_steps=4, rsqrt_mn=True)
        m2 = 0.9 * mom + (1 - 0.9) * (G + 0.1 * W)
        assert np.max(np.abs(out["mom"] - m2)) <= 1e-15
        S = np.stack([np.where(O.polar_ns(m2[p], 3) >= 0, 1, -1) for p in range(M)])
        vote = np.where(S.sum(0) >= 0, 1, -1)
        assert np.array_equal(out["vote"], vote)
        assert abs(np.linalg.norm(out["vote"]) - np.sqrt(r * c)) < 1e-12     # ||S-bar||_F = sqrt(mn)
        # local polar: same closed form on the +-1 matrix; then W - eta/sqrt(mn) D
        U, s, Vt = np.linalg.svd(vote.astype(float), full_matrices=False)
        x = s / np.sqrt(r * c)
        for _ in range(4):
            x = 1.5 * x - 0.5 * x ** 3
        D = (U * x) @ Vt
        assert np.max(np.abs(out["D"] - D)) <= 1e-12
        assert np.max(np.abs(out["W"] - (W - 1e-2 / np.sqrt(r * c) * D))) <= 1e-14
    both = [O.signmuon_step(W, mom, G, beta=0.9, lr=1e-2, ns_steps=3, sign_fmt=f)["W"]
            for f in ("1bit", "int8")]
    assert np.array_equal(both[0], both[1])               # the two transports agree


# ---------------------------------------------------------------- P13
def test_momentum_closed_form_and_float32_rounding_order():
    g = wl.rng_for(15)
    G = g.standard_normal((2, 3, 5))
    m = np.zeros_like(G)
    for t in range(1, 8):
        m = O.momentum_update(m, G, None, 0.9)
        assert np.max(np.abs(m - (1 - 0.9 ** t) * G)) <= 1e-15          # (1 - beta^t) G
    W = g.standard_normal((3, 5))
    m1 = O.momentum_update(np.ones_like(G), G, W, 0.5, weight_decay=2.0)
    assert np.max(np.abs(m1 - (0.5 + 0.5 * (G + 2.0 * W)))) <= 1e-15
    # float32 variant: each product and the sum rounded separately, 1-beta in float32
    G32, m32, W32 = G.astype(np.float32), g.standard_normal(G.shape).astype(np.float32), W.astype(np.float32)
    out = O.momentum_update(m32, G32, W32, 0.9, 0.1, dtype=np.float32)
    b, wd = np.float32(0.9), np.float32(0.1)
    omb = np.float32(np.float32(1.0) - b)
    for idx in np.ndindex(*G32.shape):
        gt = np.float32(G32[idx] + np.float32(wd * W32[idx[1:]]))
        ref = np.float32(np.float32(b * m32[idx]) + np.float32(omb * gt))
        assert out[idx] == ref
    assert out.dtype == np.float32


def test_update_rule():
    W = np.arange(12.0).reshape(3, 4)
    D = np.where(np.arange(12).reshape(3, 4) % 2 == 0, 1.0, -1.0)
    assert np.array_equal(O.apply_update(W, D, 0.5), W - 0.5 * D)
    assert np.allclose(O.apply_update(W, D, 0.5, rsqrt_mn=True), W - 0.5 / np.sqrt(12) * D, rtol=0, atol=1e-15)
    out32 = O.apply_update(W.astype(np.float32), D, 0.1, dtype=np.float32)
    assert out32.dtype == np.float32
    assert np.array_equal(out32, (W.astype(np.float32) - np.float32(0.1) * D.astype(np.float32)))


def test_float32_variant_tracks_float64():
    X = wl.normal((48, 80), stream=16)
    a = O.polar_ns(X, 5, dtype=np.float32)
    b = O.polar_ns(X, 5, dtype=np.float64)
    assert a.dtype == np.float32
    assert np.linalg.norm(a - b) / np.linalg.norm(b) < 1e-5


# ---------------------------------------------------------------- P14: normalized sign (operator-norm scaling)
def test_normalized_sign_of_rank_one_sign_matrix_is_exact():
    """S = x y^T with x, y in {-1, +1}: ||S||_op = sqrt(rc) exactly, reached by PowerIter from any start
    vector not orthogonal to y, so D = S / sqrt(rc) -- the paper's "safe upper bound" form is then tight."""
    rng = np.random.default_rng(5)
    r, c = 12, 20
    x = rng.choice([-1.0, 1.0], size=r)
    y = rng.choice([-1.0, 1.0], size=c)
    S = np.outer(x, y)
    D = O.normalized_sign(S, 2, 1e-12, rng.standard_normal(c) + 3.0 * y)
    assert np.allclose(D, S / np.sqrt(r * c), rtol=1e-12, atol=0)


def test_normalized_sign_has_operator_norm_at_least_one_and_near_one():
    """PowerIter never overestimates ||S||_op (it is a Rayleigh quotient), so ||D||_op >= 1, and after a few
    iterations on a generic +-1 matrix it is within a few percent of 1; the Frobenius bound sqrt(rc) is looser."""
    rng = np.random.default_rng(6)
    r, c = 40, 64
    S = rng.choice([-1.0, 1.0], size=(r, c))
    true = np.linalg.svd(S, compute_uv=False)[0]
    for P in (0, 2, 8):
        D = O.normalized_sign(S, P, 1e-12, rng.standard_normal(c))
        op = np.linalg.svd(D, compute_uv=False)[0]
        assert op >= 1.0 - 1e-12
        if P == 8:
            assert op <= 1.1
    assert true <= np.sqrt(r * c)


def test_step_with_normalized_sign_moves_every_entry_by_the_same_amount():
    rng = np.random.default_rng(7)
    M, r, c = 3, 8, 12
    W = rng.standard_normal((r, c))
    G = rng.standard_normal((M, r, c))
    v0 = rng.standard_normal((M, c))
    out = O.signmuon_step(W, np.zeros_like(G), G, beta=0.9, lr=0.1, ns_steps=3, v0=v0, power_iters=2, op_norm=True)
    sigma = O.power_iter(out["vote"].astype(np.float64), 2, 1e-12, v0[0])
    assert np.allclose(np.abs(W - out["W"]), 0.1 / sigma, rtol=1e-12)
    assert np.array_equal(np.sign(W - out["W"]), out["vote"])
