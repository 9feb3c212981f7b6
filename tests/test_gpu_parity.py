"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bars: bit-exact for momentum (float32, stated rounding order), sign packing,
vote, counts and the fused update; PolarNS within 2e-2 relative Frobenius error
of the float32 oracle with >= 99.9 % sign agreement on entries with
|x| > 1e-3 * max|x|.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import signmuon_oracle as O

pytestmark = pytest.mark.gpu

NS_REL_TOL = 2e-2
SIGN_AGREE = 0.999


@pytest.fixture(scope="module")
def P():
    import paper_2605_16311_amd as pkg
    return pkg


@pytest.fixture(scope="module")
def ctx(P):
    c = P.Context()
    yield c
    torch.cuda.synchronize()
    c.close()


# Settings of the context's tuning switches (GEMM tile, grouping of the K steps, storage of the s x s
# matrices) under which the Newton-Schulz and whole-step cases are repeated; "auto" is what a caller gets.
VARIANTS = {
    "auto": dict(),
    "t128-pairs-upper": dict(gemm_tile=128),
    "t256-pairs-upper": dict(gemm_tile=256),
    "t128-pairs-full": dict(gemm_tile=128, ns_store="full"),
    "t256-pairs-full": dict(gemm_tile=256, ns_store="full"),
    "t128-single-upper": dict(gemm_tile=128, ns_path="single"),
    "t256-single-upper": dict(gemm_tile=256, ns_path="single"),
    "t256-single-full": dict(gemm_tile=256, ns_path="single", ns_store="full"),
    "t128-stepwise": dict(gemm_tile=128, ns_path="stepwise"),
    "t256-stepwise": dict(gemm_tile=256, ns_path="stepwise"),
}


@pytest.fixture(scope="module", params=list(VARIANTS))
def vctx(P, request):
    c = P.Context(**VARIANTS[request.param])
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bf16_dev(a_f32):
    return dev(np.asarray(a_f32, np.float32)).bfloat16()


def bf16_host(t):
    return t.float().cpu().numpy()


def ns_check(got, ref, what=""):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    big = np.abs(ref) > 1e-3 * np.max(np.abs(ref))
    agree = np.mean((got[big] >= 0) == (ref[big] >= 0)) if big.any() else 1.0
    assert rel <= NS_REL_TOL, f"{what}: rel Frobenius {rel:.3e}"
    assert agree >= SIGN_AGREE, f"{what}: sign agreement {agree:.5f}"
    return rel, agree


# ------------------------------------------------------------------ a1
@pytest.mark.parametrize("M,r,c,wd", [(4, 256, 256, 0.0), (3, 37, 53, 0.0), (2, 64, 576, 0.1),
                                      (5, 129, 100, 0.05), (1, 1, 1, 0.0), (2, 1000, 2048, 0.0)])
def test_momentum_bit_exact(P, ctx, M, r, c, wd):
    g = wl.worker_grads("single256", 0, r, c, M=M)
    m0 = wl.normal((M, r, c), stream=21)
    w = wl.weights(r, c)
    ref = O.momentum_update(m0, g, w, 0.9, wd, dtype=np.float32)
    mom, x = dev(m0), torch.empty((M, r, c), dtype=torch.bfloat16, device="cuda")
    ss = torch.empty(M, dtype=torch.float32, device="cuda")
    P.signmuon_momentum(ctx, mom, dev(g), dev(w) if wd else None, 0.9, wd, x_bf16=x, sumsq=ss)
    got = mom.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(bf16_host(x), wl.from_bf16_bits(wl.to_bf16_bits(ref)))
    ss_ref = np.sum(ref.astype(np.float64) ** 2, axis=(1, 2))
    assert np.allclose(ss.cpu().numpy(), ss_ref, rtol=1e-5)
    # second step from the new state, no side outputs
    ref2 = O.momentum_update(ref, g, w, 0.9, wd, dtype=np.float32)
    P.signmuon_momentum(ctx, mom, dev(g), dev(w) if wd else None, 0.9, wd)
    assert np.array_equal(mom.cpu().numpy().view(np.uint32), ref2.view(np.uint32))


# ------------------------------------------------------------------ a5
@pytest.mark.parametrize("n", [1, 7, 8, 63, 64, 65, 1000, 4096, 65536 + 13, 300001])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_sign_pack_bit_exact(P, ctx, n, dt):
    batch = 3
    x = wl.normal((batch, n), stream=22, block=n)
    sv = wl.special_values_f32()
    x[0, : min(n, sv.size)] = sv[: min(n, sv.size)]
    x[1, ::3] = 0.0
    x[2, 1::5] = -0.0
    if dt == "bf16":
        xb = wl.from_bf16_bits(wl.to_bf16_bits(x))
        u = dev(wl.to_bf16_bits(x).view(np.int16)).view(torch.bfloat16)
    else:
        xb, u = x, dev(x)
    stride = O.packed_stride_bytes(n)
    out = torch.full((batch, stride + 8), 0xAA, dtype=torch.uint8, device="cuda")
    P.signmuon_sign_pack(ctx, u, "1bit", out)
    got = out.cpu().numpy()
    for b in range(batch):
        assert np.array_equal(got[b, :stride], O.pack_bits(O.sign_entries(xb[b]))), (n, dt, b)
        assert np.all(got[b, stride:] == 0xAA)          # nothing written past the row
    o8 = torch.full((batch, n + 5), 7, dtype=torch.int8, device="cuda")
    P.signmuon_sign_pack(ctx, u, "int8", o8)
    g8 = o8.cpu().numpy()
    for b in range(batch):
        assert np.array_equal(g8[b, :n], O.signs_pm1(xb[b]))
        assert np.all(g8[b, n:] == 7)


def test_sign_pack_empty_and_errors(P, ctx):
    u = torch.empty((2, 0), dtype=torch.float32, device="cuda")
    out = torch.zeros((2, 8), dtype=torch.uint8, device="cuda")
    P.signmuon_sign_pack(ctx, u, "1bit", out)
    u = torch.zeros((1, 100), dtype=torch.float32, device="cuda")
    with pytest.raises(P.SignMuonError):
        P.signmuon_sign_pack(ctx, u, "1bit", torch.zeros((1, 8), dtype=torch.uint8, device="cuda"))
    with pytest.raises(P.SignMuonError):
        P.signmuon_sign_pack(ctx, u, "int8", torch.zeros((1, 50), dtype=torch.int8, device="cuda"))


# ------------------------------------------------------------------ a6 (+ a8)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8, 16, 33, 300])
@pytest.mark.parametrize("n", [1, 5, 64, 100, 4099, 70001])
def test_vote_bit_exact(P, ctx, M, n):
    rng = wl.rng_for(23, block=M, worker=n)
    S = rng.choice(np.array([-1, 1], np.int8), size=(M, n), p=[0.45, 0.55])
    S[:, : min(n, 4)] = 1
    if M % 2 == 0 and n > 8:
        S[: M // 2, 5] = 1
        S[M // 2:, 5] = -1                                    # a forced tie
    packed = np.stack([O.pack_bits((S[p] > 0).astype(np.uint8)) for p in range(M)])
    stride = packed.shape[1]
    vote_ref, tot_ref = O.majority_vote_int8(S)
    vote1_ref, c_ref = O.majority_vote_bits(packed, M, n)
    assert np.array_equal(vote_ref, vote1_ref)
    w0 = wl.normal((n,), stream=24, block=n)
    lr = 0.01
    w_ref = O.apply_update(w0.reshape(1, n), vote_ref.reshape(1, n), lr, dtype=np.float32).reshape(n)
    for fmt, signs, counts_ref, sb in (("1bit", packed, c_ref, stride), ("int8", S, tot_ref, n)):
        d_signs = dev(signs)
        # voted bits
        vb = torch.full((stride + 8,), 0x55, dtype=torch.uint8, device="cuda")
        P.signmuon_majority_vote(ctx, d_signs, fmt, M, n, sb, voted=vb, vfmt="bits")
        g = vb.cpu().numpy()
        assert np.array_equal(g[:stride], O.pack_bits((vote_ref > 0).astype(np.uint8))), (fmt, M, n)
        assert np.all(g[stride:] == 0x55)
        # expanded formats + counts + fused update, one call each
        cnt = torch.full((n + 4,), -7, dtype=torch.int32, device="cuda")
        w = dev(np.concatenate([w0, np.full(4, 3.0, np.float32)]))
        v8 = torch.full((n + 4,), 9, dtype=torch.int8, device="cuda")
        P.signmuon_majority_vote(ctx, d_signs, fmt, M, n, sb, voted=v8, vfmt="int8", counts=cnt, w=w, lr_scaled=lr)
        assert np.array_equal(v8.cpu().numpy()[:n], vote_ref) and np.all(v8.cpu().numpy()[n:] == 9)
        assert np.array_equal(cnt.cpu().numpy()[:n], counts_ref) and np.all(cnt.cpu().numpy()[n:] == -7)
        gw = w.cpu().numpy()
        assert np.array_equal(gw[:n].view(np.uint32), w_ref.view(np.uint32)) and np.all(gw[n:] == 3.0)
        vb16 = torch.zeros((n + 4,), dtype=torch.bfloat16, device="cuda")
        P.signmuon_majority_vote(ctx, d_signs, fmt, M, n, sb, voted=vb16, vfmt="bf16")
        assert np.array_equal(bf16_host(vb16)[:n], vote_ref.astype(np.float32)) and np.all(bf16_host(vb16)[n:] == 0)
        vf = torch.zeros((n + 4,), dtype=torch.float32, device="cuda")
        P.signmuon_majority_vote(ctx, d_signs, fmt, M, n, sb, voted=vf, vfmt="f32")
        assert np.array_equal(vf.cpu().numpy()[:n], vote_ref.astype(np.float32)) and np.all(vf.cpu().numpy()[n:] == 0)


@pytest.mark.parametrize("M", [1, 2, 3, 7, 8, 31, 32, 100, 255, 256])
@pytest.mark.parametrize("n", [32, 64 * 37, 32 * 2049, 256 * 300 + 32])
def test_vote_word_aligned_without_counts(P, ctx, M, n):
    """n % 32 == 0, no counts: the form the step uses (bit-sliced counting, one thread per 32-bit word);
    voted bf16 and the fused update in one call, against the scalar definition (eq. mv_def)."""
    rng = wl.rng_for(27, block=M, worker=n)
    S = rng.choice(np.array([-1, 1], np.int8), size=(M, n), p=[0.5, 0.5])
    if M % 2 == 0:
        S[: M // 2, 3::17] = 1
        S[M // 2:, 3::17] = -1                                # forced ties -> +1
    packed = np.stack([O.pack_bits((S[p] > 0).astype(np.uint8)) for p in range(M)])
    stride = packed.shape[1]
    vote_ref, _ = O.majority_vote_int8(S)
    w0 = wl.normal((n,), stream=28, block=n)
    lr = 0.0625
    w_ref = O.apply_update(w0.reshape(1, n), vote_ref.reshape(1, n), lr, dtype=np.float32).reshape(n)
    w = dev(np.concatenate([w0, np.full(8, 3.0, np.float32)]))
    vb16 = torch.full((n + 8,), 5.0, dtype=torch.bfloat16, device="cuda")
    P.signmuon_majority_vote(ctx, dev(packed), "1bit", M, n, stride, voted=vb16, vfmt="bf16", w=w, lr_scaled=lr)
    gv = bf16_host(vb16)
    assert np.array_equal(gv[:n], vote_ref.astype(np.float32)) and np.all(gv[n:] == 5.0), (M, n)
    gw = w.cpu().numpy()
    assert np.array_equal(gw[:n].view(np.uint32), w_ref.view(np.uint32)) and np.all(gw[n:] == 3.0), (M, n)


@pytest.mark.parametrize("M", [1, 2, 16, 127, 300])
@pytest.mark.parametrize("n", [16, 4096, 65536 + 16])
def test_vote_int8_sixteen_entry_groups(P, ctx, M, n):
    """int8 signs with n % 16 == 0 and aligned rows (one thread per 16 entries): int32 sums, voted int8 and
    bf16, fused update, against the scalar definition; sums beyond the int8 range at M = 300."""
    rng = wl.rng_for(30, block=M, worker=n)
    S = rng.choice(np.array([-1, 1], np.int8), size=(M, n), p=[0.5, 0.5])
    if M % 2 == 0:
        S[: M // 2, 1::13] = 1
        S[M // 2:, 1::13] = -1                                # forced ties -> +1
    S[:, 0] = 1                                               # sum = M (overflows int8 at M = 300)
    vote_ref, tot_ref = O.majority_vote_int8(S)
    w0 = wl.normal((n,), stream=31, block=n)
    lr = 0.03125
    w_ref = O.apply_update(w0.reshape(1, n), vote_ref.reshape(1, n), lr, dtype=np.float32).reshape(n)
    d_signs = dev(S)
    cnt = torch.full((n + 16,), -7, dtype=torch.int32, device="cuda")
    w = dev(np.concatenate([w0, np.full(16, 3.0, np.float32)]))
    v8 = torch.full((n + 16,), 9, dtype=torch.int8, device="cuda")
    P.signmuon_majority_vote(ctx, d_signs, "int8", M, n, n, voted=v8, vfmt="int8", counts=cnt, w=w, lr_scaled=lr)
    assert np.array_equal(v8.cpu().numpy()[:n], vote_ref) and np.all(v8.cpu().numpy()[n:] == 9)
    assert np.array_equal(cnt.cpu().numpy()[:n], tot_ref) and np.all(cnt.cpu().numpy()[n:] == -7)
    gw = w.cpu().numpy()
    assert np.array_equal(gw[:n].view(np.uint32), w_ref.view(np.uint32)) and np.all(gw[n:] == 3.0)
    vb16 = torch.full((n + 16,), 5.0, dtype=torch.bfloat16, device="cuda")
    P.signmuon_majority_vote(ctx, d_signs, "int8", M, n, n, voted=vb16, vfmt="bf16")
    gv = bf16_host(vb16)
    assert np.array_equal(gv[:n], vote_ref.astype(np.float32)) and np.all(gv[n:] == 5.0)


@pytest.mark.parametrize("snr", [0.25, 1.0])
def test_majority_vote_sign_error_falls_like_inverse_sqrt_m(P, ctx, snr):
    """Lemma "Majority vote improves sign reliability": with M independent workers whose gradient entries are
    g + sigma z (symmetric unimodal noise), the vote's sign-error rate is at most sigma / (sqrt(M) |g|).  The
    library's pack + vote on synthetic entries: the measured rate matches the exact binomial value (ties -> +1),
    obeys the bound and falls with M."""
    from scipy import stats
    n = 1 << 20
    g = np.where(np.arange(n) % 2 == 0, snr, -snr).astype(np.float32)      # sigma = 1
    prev = 1.0
    p1 = float(stats.norm.cdf(-snr))                                       # one worker's failure probability
    for M in (1, 4, 16, 64):
        z = wl.normal((M, n), stream=32, block=M, worker=int(snr * 100))
        u = dev((g[None, :] + z).astype(np.float32))
        stride = O.packed_stride_bytes(n)
        bits = torch.zeros((M, stride), dtype=torch.uint8, device="cuda")
        P.signmuon_sign_pack(ctx, u, "1bit", bits)
        v8 = torch.zeros((n,), dtype=torch.int8, device="cuda")
        P.signmuon_majority_vote(ctx, bits, "1bit", M, n, stride, voted=v8, vfmt="int8")
        vote = v8.cpu().numpy()
        fail = float(np.mean(vote != np.sign(g)))
        # exact: entries with g > 0 fail iff fewer than M/2 workers are right; with g < 0 a tie also fails
        k = np.arange(M + 1)
        pmf = stats.binom.pmf(k, M, 1.0 - p1)                              # number of correct workers
        q_pos = pmf[2 * k < M].sum()
        q_neg = pmf[2 * k <= M].sum()
        q = 0.5 * (q_pos + q_neg)
        assert abs(fail - q) <= 5.0 * np.sqrt(q * (1 - q) / n) + 1e-6, (M, fail, q)
        assert fail <= 1.0 / (np.sqrt(M) * snr) + 1e-3, (M, fail)
        assert fail < prev or M == 1
        prev = fail


def test_vote_ignores_garbage_tail_bits_and_dropped_worker(P, ctx):
    M, n = 5, 70
    rng = wl.rng_for(25)
    S = rng.choice(np.array([-1, 1], np.int8), size=(M, n))
    packed = np.stack([O.pack_bits((S[p] > 0).astype(np.uint8)) for p in range(M)])
    ref, _ = O.majority_vote_int8(S)
    dirty = packed.copy()
    dirty[:, n // 8] |= np.uint8(0xFF << (n % 8) & 0xFF)      # set padding bits in every worker
    dirty[:, n // 8 + 1:] = 0xFF
    vb = torch.zeros((16,), dtype=torch.uint8, device="cuda")
    P.signmuon_majority_vote(ctx, dev(dirty), "1bit", M, n, 16, voted=vb, vfmt="bits")
    assert np.array_equal(vb.cpu().numpy(), O.pack_bits((ref > 0).astype(np.uint8)))
    # a dropped worker: vote over the first M-1 rows only
    ref4, _ = O.majority_vote_int8(S[:4])
    P.signmuon_majority_vote(ctx, dev(packed), "1bit", 4, n, 16, voted=vb, vfmt="bits")
    assert np.array_equal(vb.cpu().numpy(), O.pack_bits((ref4 > 0).astype(np.uint8)))


# ------------------------------------------------------------------ a2-a4
NS_CASES = [
    # (batch, rows, cols, steps, scale, coeffs)
    (4, 256, 256, 5, "fro", O.PAPER_COEFFS),
    (2, 64, 576, 5, "fro", O.PAPER_COEFFS),
    (2, 576, 64, 5, "fro", O.PAPER_COEFFS),
    (3, 128, 320, 3, "fro", O.PAPER_COEFFS),
    (2, 200, 136, 5, "fro", O.PAPER_COEFFS),        # padding in both dimensions, tall
    (2, 100, 333, 4, "fro", O.PAPER_COEFFS),        # padding, wide, odd sizes
    (1, 512, 1152, 5, "fro", O.PAPER_COEFFS),
    (2, 256, 256, 1, "fro", O.PAPER_COEFFS),
    (2, 192, 448, 0, "fro", O.PAPER_COEFFS),        # K = 0: only the scaling
    (2, 256, 384, 5, "spectral", O.PAPER_COEFFS),
    (2, 384, 256, 5, "spectral", O.PAPER_COEFFS),
    (2, 128, 128, 4, "none", O.PAPER_COEFFS),
    (2, 192, 320, 3, "fro", (2.0, -1.5, 0.5)),      # quintic polynomial (step-by-step form)
    (2, 192, 320, 4, "fro", (1.6, -0.6, 0.0)),      # cubic with a > 3/2 (step-by-step form)
    (2, 256, 640, 2, "fro", O.PAPER_COEFFS),        # shortest short-side recurrence
    (2, 320, 192, 7, "fro", O.PAPER_COEFFS),        # two segments (5 + 2), tall
    (2, 256, 640, 10, "fro", O.PAPER_COEFFS),       # two full segments, wide
    (1, 512, 512, 10, "spectral", O.PAPER_COEFFS),  # square, near convergence
    (2, 136, 200, 6, "fro", O.PAPER_COEFFS),        # padding + two segments (5 + 1)
    (2, 192, 448, 8, "fro", O.PAPER_COEFFS),        # segments 5 + 3: two steps at a time, then one
    (2, 448, 192, 9, "fro", O.PAPER_COEFFS),        # segments 5 + 4: two pairs, tall
    (2, 256, 384, 5, "fro", (1.25, -0.4, 0.0)),     # another cubic on the short-side recurrence
    (2, 256, 384, 4, "none", (1.4, -0.45, 0.0)),
    (2, 320, 512, 5, "fro", O.PAPER_COEFFS),        # short side 320: a whole and a partial 256-block
    (1, 640, 576, 5, "fro", O.PAPER_COEFFS),        # short side 576 (tall): three blocks, the last partial
    (1, 640, 640, 4, "fro", O.PAPER_COEFFS),        # square, 2.5 blocks
]


@pytest.mark.parametrize("batch,r,c,steps,scale,coeffs", NS_CASES)
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_polar_ns_against_fp32_oracle(P, vctx, batch, r, c, steps, scale, coeffs, dt):
    ctx = vctx
    x = wl.normal((batch, r, c), stream=26, block=r, worker=c)
    if scale == "none":
        x = x / (1.05 * np.linalg.norm(x, ord=2, axis=(1, 2), keepdims=True)).astype(np.float32)
    v0 = wl.start_vectors(batch, c, block=r)
    if dt == "bf16":
        xin = wl.from_bf16_bits(wl.to_bf16_bits(x))
        xd = dev(wl.to_bf16_bits(x).view(np.int16)).view(torch.bfloat16)
    else:
        xin, xd = x, dev(x)
    P.signmuon_polar_ns(ctx, xd, steps, coeffs=coeffs, scale=scale, power_iters=2, eps=1e-12,
                        v0=dev(v0) if scale == "spectral" else None)
    got = xd.float().cpu().numpy()
    for b in range(batch):
        ref = O.polar_ns(xin[b], steps, coeffs, scale, 2, 1e-12, v0[b], dtype=np.float32)
        ns_check(got[b], ref, f"{(batch, r, c, steps, scale, dt)} item {b}")


@pytest.mark.parametrize("opts", [dict(gemm_tile=128), dict(gemm_tile=256), dict(gemm_tile=256, ns_store="full"),
                                  dict(gemm_tile=128, ns_path="stepwise")])
@pytest.mark.parametrize("r,c", [(1152, 1408), (1408, 1152)])
def test_polar_ns_on_grids_of_several_tile_bands(P, opts, r, c):
    """The GEMM kernels list a matrix's tiles in bands of 4 (256-wide tiles) or 8 (128-wide) tile rows.  A short
    side of 1152 is 4.5 and 9 tiles: the symmetric products and the apply run over a full band and a ragged
    one, in both operand orientations."""
    ctx = P.Context(**opts)
    x = wl.normal((2, r, c), stream=27, block=r, worker=c)
    xd = dev(wl.to_bf16_bits(x).view(np.int16)).view(torch.bfloat16)
    xin = wl.from_bf16_bits(wl.to_bf16_bits(x))
    P.signmuon_polar_ns(ctx, xd, 5, scale="fro")
    got = xd.float().cpu().numpy()
    for b in range(2):
        ns_check(got[b], O.polar_ns(xin[b], 5, O.PAPER_COEFFS, "fro", 2, 1e-12, None, dtype=np.float32),
                 f"{(r, c, opts)} item {b}")
    torch.cuda.synchronize()
    ctx.close()


def test_polar_ns_zero_matrix_and_errors(P, ctx):
    x = torch.zeros((2, 64, 128), dtype=torch.float32, device="cuda")
    P.signmuon_polar_ns(ctx, x, 5)
    assert torch.all(x == 0) and not torch.isnan(x).any()
    with pytest.raises(P.SignMuonError):
        P.signmuon_polar_ns(ctx, x, 5, scale="spectral")          # no v0
    with pytest.raises(P.SignMuonError):
        P.signmuon_polar_ns(ctx, x, -1)


# ------------------------------------------------------------------ whole step
def run_step_case(P, ctx, shapes, M, *, sign_fmt, Kp, K=5, scale="fro", wd=0.0, rsqrt=False, stream=31,
                  grads=None, check_ns_blocks=None):
    n = len(shapes)
    lr, beta = 1e-3, 0.9
    W0 = [wl.weights(r, c, block=i, stream=stream) for i, (r, c) in enumerate(shapes)]
    G = grads or [wl.normal((M, r, c), stream=stream, block=i, worker=7) for i, (r, c) in enumerate(shapes)]
    M0 = [0.1 * wl.normal((M, r, c), stream=stream, block=i, worker=8) for i, (r, c) in enumerate(shapes)]
    V0 = [wl.start_vectors(M, c, block=i, stream=stream) for i, (r, c) in enumerate(shapes)]
    w = [dev(a) for a in W0]
    mom = [dev(a) for a in M0]
    grad = [dev(a) for a in G]
    v0 = [dev(a) for a in V0] if scale == "spectral" else None
    d = [r * c for r, c in shapes]
    sstride = [O.packed_stride_bytes(x) if sign_fmt == "1bit" else x for x in d]
    signs = [torch.zeros((M, s), dtype=torch.uint8, device="cuda") for s in sstride]
    counts = [torch.zeros((x,), dtype=torch.int32, device="cuda") for x in d]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, weight_decay=wd, scale=scale, v0=v0,
                      sign_fmt=sign_fmt, local_polar_steps=Kp, update_rsqrt_mn=rsqrt,
                      signs_out=signs, counts_out=counts, u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    for i, (r, c) in enumerate(shapes):
        # a1: momentum bit-exact
        m_ref = O.momentum_update(M0[i], G[i], W0[i], beta, wd, dtype=np.float32)
        assert np.array_equal(mom[i].cpu().numpy().view(np.uint32), m_ref.view(np.uint32)), f"momentum block {i}"
        U = bf16_host(u_out[i])
        # a2-a4: U against the float32 oracle (on selected blocks: it is the slow part)
        if check_ns_blocks is None or i in check_ns_blocks:
            for p in range(M):
                ref = O.polar_ns(m_ref[p], K, O.PAPER_COEFFS, scale, 2, 1e-12, V0[i][p], dtype=np.float32)
                ns_check(U[p], ref, f"U block {i} worker {p}")
        # a5: the oracle's packing of the GPU's own U, bit-exact
        if sign_fmt == "1bit":
            s_ref = np.stack([O.pack_bits(O.sign_entries(U[p])) for p in range(M)])
            vote_ref, c_ref = O.majority_vote_bits(s_ref, M, d[i])
        else:
            s_ref = np.stack([O.signs_pm1(U[p]).reshape(-1) for p in range(M)]).view(np.uint8)
            vote_ref, c_ref = O.majority_vote_int8(s_ref.view(np.int8))
        assert np.array_equal(signs[i].cpu().numpy(), s_ref), f"signs block {i}"
        # a6: vote / counts of those signs, bit-exact
        assert np.array_equal(counts[i].cpu().numpy(), c_ref), f"counts block {i}"
        S_bar = vote_ref.reshape(r, c)
        D = bf16_host(d_out[i])
        if Kp == 0:
            assert np.array_equal(D, S_bar.astype(np.float32)), f"vote block {i}"
        elif check_ns_blocks is None or i in check_ns_blocks:
            # a7: local polar of the voted matrix against the float32 oracle
            ref = O.local_polar(S_bar, Kp, O.PAPER_COEFFS, scale, 2, 1e-12, V0[i][0], dtype=np.float32)
            ns_check(D, ref, f"D block {i}")
        # a8: W - step * D with the GPU's own D, bit-exact
        w_ref = O.apply_update(W0[i], D, lr, rsqrt, dtype=np.float32)
        assert np.array_equal(w[i].cpu().numpy().view(np.uint32), w_ref.view(np.uint32)), f"W block {i}"
    return plan


def test_step_single256(P, vctx):
    """256x256, M=4, N(0,1) gradients from zero momentum, 5 NS steps, 1-bit, no local polar."""
    ctx = vctx
    cfg = wl.WORKLOADS["single256"]
    shapes, M = cfg["shapes"], cfg["M"]
    G = [wl.worker_grads("single256", 0, 256, 256)]
    run_step_case(P, ctx, shapes, M, sign_fmt="1bit", Kp=0, grads=G)


@pytest.mark.parametrize("sign_fmt", ["1bit", "int8"])
@pytest.mark.parametrize("Kp", [0, 3])
def test_step_mixed_set(P, vctx, sign_fmt, Kp):
    ctx = vctx
    # (200, 160) and (96, 224): signs packed by the apply GEMM with zero padding in both dimensions;
    # (100, 72): rows that do not pack into whole words (separate sign-pack launch)
    shapes = [(64, 192), (192, 64), (64, 192), (128, 128), (100, 72), (64, 192), (200, 160), (96, 224)]
    run_step_case(P, ctx, shapes, 3, sign_fmt=sign_fmt, Kp=Kp, wd=0.1, rsqrt=(Kp > 0))


@pytest.mark.parametrize("special", [False, True])
def test_step_signs_written_by_the_apply_alone(P, vctx, special):
    """Without a u_out tap the last apply writes only the packed signs (U is never stored; the bits come
    straight from the accumulators).  The same step with all taps (checked against the oracle by the cases
    above; there the signs are taken from the stored bf16 U) must give the same signs, counts and W.
    special: a column of entries near the bottom of the fp32 range (its outputs fall among the
    denormals, negative ones included), a NaN (the whole matrix turns NaN: all signs -1) and a zero matrix."""
    # (64, 100) cannot be packed by the GEMM; (200, 160) is packed with padding in both dimensions;
    # (320, 576) and (576, 320) span two tiles of 256 each way with a ragged second tile
    ctx = vctx
    shapes, M = [(128, 256), (256, 128), (192, 192), (64, 100), (200, 160), (320, 576), (576, 320)], 3
    outs = []
    for tapped in (True, False):
        w = [dev(wl.weights(r, c, block=i)) for i, (r, c) in enumerate(shapes)]
        mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
        g_host = [wl.normal((M, r, c), stream=29, block=i) for i, (r, c) in enumerate(shapes)]
        if special:
            sgn = np.where(wl.normal((M, 128), stream=30) >= 0, 1.0, -1.0).astype(np.float32)
            g_host[0][:, :, 5] = sgn * np.float32(3e-37)
            g_host[1][0, 7, 9] = np.float32("nan")
            g_host[2][1] = 0.0
            sgn = np.where(wl.normal((M, 320), stream=35) >= 0, 1.0, -1.0).astype(np.float32)
            g_host[5][:, :, 300] = sgn * np.float32(3e-37)          # a column in the second 256-tile
            g_host[6][2, 400, 17] = np.float32("nan")
        grad = [dev(g) for g in g_host]
        d = [r * c for r, c in shapes]
        signs = [torch.zeros((M, O.packed_stride_bytes(x)), dtype=torch.uint8, device="cuda") for x in d]
        counts = [torch.zeros((x,), dtype=torch.int32, device="cuda") for x in d]
        u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes] if tapped else None
        plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-2, ns_steps=5, sign_fmt="1bit", local_polar_steps=2,
                          signs_out=signs, counts_out=counts, u_out=u_out)
        P.signmuon_step(ctx, plan)
        torch.cuda.synchronize()
        outs.append(([t.cpu().numpy() for t in signs], [t.cpu().numpy() for t in counts], [t.cpu().numpy() for t in w]))
    for a, b in zip(outs[0], outs[1]):
        for x, y in zip(a, b):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8))


def test_step_replays_from_a_hip_graph(P):
    """After the first call (which plans and clears the workspace) a step only enqueues kernels on the
    context's stream, so it can be captured once and replayed.  Four replays, with eager work and
    synchronisations between them, must leave W and the momentum bit-identical to four eager steps."""
    shapes, M = [(128, 256), (256, 128), (192, 192), (64, 100)], 3

    def fresh():
        w = [dev(wl.weights(r, c, block=i, stream=33)) for i, (r, c) in enumerate(shapes)]
        mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
        grad = [dev(wl.normal((M, r, c), stream=33, block=i)) for i, (r, c) in enumerate(shapes)]
        return w, mom, grad

    results = []
    for use_graph in (False, True):
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            w, mom, grad = fresh()
            ctx = P.Context(stream=side)
            plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-2, ns_steps=5, sign_fmt="1bit", local_polar_steps=3)
            P.signmuon_step(ctx, plan)                      # plans the workspace
            side.synchronize()
            snaps = []
            if use_graph:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    P.signmuon_step(ctx, plan)
            for rep in range(4):
                if use_graph:
                    graph.replay()
                else:
                    P.signmuon_step(ctx, plan)
                torch.cuda.synchronize()
                scratch = torch.randn((1 << 16,), device="cuda").sum().item()      # unrelated eager work between replays
                assert np.isfinite(scratch)
                snaps.append(([t.cpu().numpy().copy() for t in w], [t.cpu().numpy().copy() for t in mom]))
            ctx.close()
        results.append(snaps)
    for rep in range(4):
        for a, b in zip(results[0][rep][0] + results[0][rep][1], results[1][rep][0] + results[1][rep][1]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"replay {rep}"


def test_step_with_normalized_sign_update(P, ctx):
    """update scale mode 2: W <- W - lr S / max(PowerIter(S), eps) with S the voted sign (the appendix's
    "normalized sign").  The vote is checked bit-exactly from the GPU's own U; the step size, which every entry
    of a block shares, against the float32 oracle's PowerIter on the same S and start vector."""
    shapes, M, lr = [(128, 256), (200, 160), (64, 100), (256, 128)], 3, 0.05
    W0 = [wl.weights(r, c, block=i, stream=34) for i, (r, c) in enumerate(shapes)]
    G = [wl.normal((M, r, c), stream=34, block=i) for i, (r, c) in enumerate(shapes)]
    V0 = [wl.start_vectors(M, c, block=i, stream=34) for i, (r, c) in enumerate(shapes)]
    w = [dev(a) for a in W0]
    mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
    grad = [dev(a) for a in G]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=0.9, lr=lr, ns_steps=3, power_iters=2, v0=[dev(a) for a in V0],
                      update_rsqrt_mn="op_norm", u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    for i, (r, c) in enumerate(shapes):
        U = u_out[i].float().cpu().numpy()
        signs = np.stack([O.pack_bits(O.sign_entries(U[p])) for p in range(M)])
        vote, _ = O.majority_vote_bits(signs, M, r * c)
        S = vote.reshape(r, c).astype(np.float32)
        assert np.array_equal(d_out[i].float().cpu().numpy(), S)
        moved = (W0[i].astype(np.float64) - w[i].cpu().numpy().astype(np.float64)) * S      # = step, entry by entry
        step_ref = lr / float(O.power_iter(S, 2, 1e-12, V0[i][0]))
        assert abs(moved.mean() - step_ref) <= 1e-3 * step_ref, (i, moved.mean(), step_ref)
        assert np.all(np.abs(moved - moved.mean()) <= 2e-3 * step_ref)                      # one step size per block
    with pytest.raises(P.SignMuonError):                                                    # not with a local polar step
        P.signmuon_step(ctx, P.StepPlan(w, mom, grad, beta=0.9, lr=lr, ns_steps=3, v0=[dev(a) for a in V0],
                                        update_rsqrt_mn="op_norm", local_polar_steps=2))


def test_step_spectral(P, vctx):
    run_step_case(P, vctx, [(128, 256), (256, 128)], 2, sign_fmt="1bit", Kp=2, scale="spectral")


@pytest.mark.parametrize("mode", ["fused", "separate", "auto"])
def test_step_spectral_power_iteration_forms(P, mode):
    """Alg. PowerIter over a set that spans every form: matrices for each column-strip count of the fused pass
    (one read of X for X v and X^T u), one too wide for it (a pass per product), ragged row chunks and padding."""
    shapes = [(72, 4608), (200, 160), (96, 1800), (130, 2304), (64, 3000), (70, 4000), (300, 64)]
    ctx = P.Context(power_iter=mode)
    run_step_case(P, ctx, shapes, 2, sign_fmt="1bit", Kp=1, K=3, scale="spectral", stream=37)
    torch.cuda.synchronize()
    ctx.close()


def test_nan_worker_on_a_padded_shape_does_not_leak_into_other_blocks(P):
    """A NaN in one worker's gradient turns that worker's whole matrix NaN (every sign -1), zero padding of its
    slots in the working layout included.  After the vote those slots hold other blocks' voted matrices, so
    the padding is cleared again: the blocks without a NaN worker must come out exactly as in a run where
    the NaN is replaced by an ordinary number.  200 x 160 pads both dimensions; K = 7 makes both working
    buffers carry apply outputs; the local polar step reads the voted matrices with their padding."""
    shapes, M = [(200, 160)] * 3 + [(136, 200)] * 2, 3

    def run(ctx, poisoned):
        G = [wl.normal((M, r, c), stream=36, block=i) for i, (r, c) in enumerate(shapes)]
        if poisoned:
            G[0][1, 3, 4] = np.float32("nan")
            G[3][2, 100, 150] = np.float32("inf")
        w = [dev(wl.weights(r, c, block=i, stream=36)) for i, (r, c) in enumerate(shapes)]
        mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
        d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
        plan = P.StepPlan(w, mom, [dev(g) for g in G], beta=0.9, lr=1e-2, ns_steps=7, local_polar_steps=3, d_out=d_out)
        P.signmuon_step(ctx, plan)
        torch.cuda.synchronize()
        return [t.cpu().numpy() for t in w], [bf16_host(t) for t in d_out]

    c0 = P.Context()
    w_ref, d_ref = run(c0, False)
    c0.close()
    c1 = P.Context()
    w_bad, d_bad = run(c1, True)
    w_after, d_after = run(c1, False)          # the same context, after it has seen the NaN
    c1.close()
    for i in range(len(shapes)):
        assert np.isfinite(w_ref[i]).all() and np.isfinite(d_ref[i]).all()
        assert np.array_equal(w_after[i], w_ref[i]) and np.array_equal(d_after[i], d_ref[i]), f"block {i} after the NaN"
    for i in (1, 2, 4):                        # blocks whose workers are all finite
        assert np.array_equal(w_bad[i], w_ref[i]) and np.array_equal(d_bad[i], d_ref[i]), f"block {i} beside the NaN"
    for i in (0, 3):                           # the vote tolerates the non-finite worker (its signs are all -1)
        assert np.isfinite(w_bad[i]).all() and np.isfinite(d_bad[i]).all()


def test_step_signsgd_limit_and_zero_gradients(P, ctx):
    # K = 0, beta = 0, M = 1: W - lr * sign(G)
    r, c = 48, 80
    G = wl.normal((1, r, c), stream=32)
    W0 = wl.weights(r, c, stream=32)
    w, mom, grad = [dev(W0)], [torch.zeros((1, r, c), device="cuda")], [dev(G)]
    plan = P.StepPlan(w, mom, grad, beta=0.0, lr=0.25, ns_steps=0)
    P.signmuon_step(ctx, plan)
    ref = O.signmuon_step(W0, np.zeros_like(G), G, beta=0.0, lr=0.25, ns_steps=0, dtype=np.float32)
    assert np.array_equal(w[0].cpu().numpy(), ref["W"])
    # all-zero gradients from zero state: every sign bit is 1, W decreases by lr
    w = [torch.ones((r, c), device="cuda")]
    z = [torch.zeros((3, r, c), device="cuda")]
    plan = P.StepPlan(w, [z[0].clone()], z, beta=0.9, lr=0.5, ns_steps=5)
    P.signmuon_step(ctx, plan)
    assert torch.all(w[0] == 0.5)


def test_step_is_deterministic_and_repeatable(P, ctx):
    shapes, M = [(128, 256), (256, 128)], 4
    outs = []
    for _ in range(2):
        W0 = [wl.weights(r, c, block=i, stream=33) for i, (r, c) in enumerate(shapes)]
        w = [dev(a) for a in W0]
        mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
        grad = [dev(wl.normal((M, r, c), stream=33, block=i)) for i, (r, c) in enumerate(shapes)]
        plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-2, ns_steps=5, local_polar_steps=2)
        for _ in range(3):
            P.signmuon_step(ctx, plan)
        outs.append([t.cpu().numpy() for t in w + mom])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
