"""GPU parity at the benchmark's full sizes and launch configuration, plus edge shapes.

The nanoGPT-124M-shaped step is run exactly as bench.py runs it (same StepPlan, grouped launches,
256 x 256 GEMM tiles), with every intermediate tapped.  Bit-exact stages are checked on ALL blocks and
workers; Newton-Schulz outputs are checked against the float32 oracle on one (block, worker) per
distinct shape, and by properties that hold at any size on the rest.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import signmuon_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2605_16311_amd as pkg
    return pkg


def rel_and_agree(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    big = np.abs(ref) > 1e-3 * np.max(np.abs(ref))
    return rel, float(np.mean((got[big] >= 0) == (ref[big] >= 0)))


def report_margins(name, rels, agrees, what):
    """Measured distance to the Newton-Schulz bar (2e-2, 99.9 %), printed so a run with -s records it."""
    if rels:
        print(f"[margin] {name} {what}: max rel Frobenius {max(rels):.3e}, min sign agreement {min(agrees):.5f} "
              f"over {len(rels)} matrices", flush=True)


def full_step_check(P, name, ns_blocks, **ctx_opts):
    import bench
    cfg, w, mom, grad = bench.make_inputs(name, torch, torch.device("cuda:0"))
    shapes, M = cfg["shapes"], cfg["M"]
    K, Kp, fmt = cfg["ns_steps"], cfg["local_polar_steps"], cfg["sign_fmt"]
    scale = cfg.get("scale", "fro")
    lr, beta = 1e-3, 0.9
    W0 = [t.cpu().numpy() for t in w]
    G = [t.cpu().numpy() for t in grad]
    V0 = [wl.start_vectors(M, c, block=i, stream=cfg["stream"]) for i, (r, c) in enumerate(shapes)]
    v0 = [torch.from_numpy(a).cuda() for a in V0] if scale == "spectral" else None
    # one warm step so the momentum is not the trivial (1 - beta) G
    ctx = P.Context(**ctx_opts)
    rels_u, agrees_u, rels_d, agrees_d = [], [], [], []
    rank_ratio = 0.0
    plan0 = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, sign_fmt=fmt, local_polar_steps=Kp, scale=scale,
                       power_iters=2, v0=v0)
    P.signmuon_step(ctx, plan0)
    torch.cuda.synchronize()
    M1 = [t.cpu().numpy() for t in mom]
    W1 = [t.cpu().numpy() for t in w]
    d = [r * c for r, c in shapes]
    stride = [O.packed_stride_bytes(x) if fmt == "1bit" else x for x in d]
    signs = [torch.zeros((M, s), dtype=torch.uint8, device="cuda") for s in stride]
    counts = [torch.zeros((x,), dtype=torch.int32, device="cuda") for x in d]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, sign_fmt=fmt, local_polar_steps=Kp, scale=scale,
                      power_iters=2, v0=v0, signs_out=signs, counts_out=counts, u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    for i, (r, c) in enumerate(shapes):
        m_ref = O.momentum_update(M1[i], G[i], None, beta, 0.0, dtype=np.float32)
        assert np.array_equal(mom[i].cpu().numpy().view(np.uint32), m_ref.view(np.uint32)), f"momentum block {i}"
        U = u_out[i].float().cpu().numpy()
        assert np.isfinite(U).all()
        # a property that holds at any size: the cubic map 1.5 x - 0.5 x^3 takes every singular value in
        # (0, sqrt(3)) into (0, 1], so after at least one step ||U||_F^2 <= min(r, c) both from a Frobenius-scaled
        # start (x <= 1) and from a power-iteration scale, which underestimates the largest singular value by
        # far less than sqrt(3); 2 % covers the bf16 rounding (measured: at most 1.001)
        fro2 = np.sum(U.astype(np.float64) ** 2, axis=(1, 2))
        rank_ratio = max(rank_ratio, float(fro2.max()) / min(r, c))
        assert np.all(fro2 <= min(r, c) * 1.02), f"block {i}: ||U||_F^2 {fro2.max()} > rank bound"
        if i in ns_blocks:
            for p in (0, M - 1):
                ref = O.polar_ns(m_ref[p], K, scale=scale, power_iters=2, v0=V0[i][p], dtype=np.float32)
                rel, agree = rel_and_agree(U[p], ref)
                rels_u.append(rel)
                agrees_u.append(agree)
                assert rel <= 2e-2 and agree >= 0.999, f"U block {i} worker {p}: rel {rel:.3e} agree {agree:.5f}"
        if fmt == "1bit":
            s_ref = np.stack([O.pack_bits(O.sign_entries(U[p])) for p in range(M)])
            vote_ref, c_ref = O.majority_vote_bits(s_ref, M, d[i])
        else:
            s_ref = np.stack([O.signs_pm1(U[p]).reshape(-1) for p in range(M)])
            vote_ref, c_ref = O.majority_vote_int8(s_ref)
            s_ref = s_ref.view(np.uint8)
        assert np.array_equal(signs[i].cpu().numpy(), s_ref), f"signs block {i}"
        assert np.array_equal(counts[i].cpu().numpy(), c_ref), f"counts block {i}"
        D = d_out[i].float().cpu().numpy()
        S_bar = vote_ref.reshape(r, c)
        if Kp == 0:
            assert np.array_equal(D, S_bar.astype(np.float32))
        else:
            assert np.sum(D.astype(np.float64) ** 2) <= min(r, c) * 1.02
            if i in ns_blocks:
                ref = O.local_polar(S_bar, Kp, scale=scale, power_iters=2, v0=V0[i][0], dtype=np.float32)
                rel, agree = rel_and_agree(D, ref)
                rels_d.append(rel)
                agrees_d.append(agree)
                assert rel <= 2e-2 and agree >= 0.999, f"D block {i}: rel {rel:.3e} agree {agree:.5f}"
        w_ref = O.apply_update(W1[i], D, lr, False, dtype=np.float32)
        assert np.array_equal(w[i].cpu().numpy().view(np.uint32), w_ref.view(np.uint32)), f"W block {i}"
    report_margins(name, rels_u, agrees_u, "U vs float32 oracle")
    report_margins(name, rels_d, agrees_d, "D (local polar) vs float32 oracle")
    print(f"[margin] {name} ({scale} scale): max ||U||_F^2 / min(r, c) = {rank_ratio:.4f}", flush=True)
    # The configuration the benchmark times has no u_out tap: the last apply then writes only the packed signs,
    # straight from its accumulators, and U is never stored.  Same state, same inputs, no U tap: the signs, the
    # counts and W must be those of the tapped step (which the oracle has just confirmed), bit for bit.
    g_signs = [t.cpu().numpy() for t in signs]
    g_counts = [t.cpu().numpy() for t in counts]
    g_w = [t.cpu().numpy() for t in w]
    for i in range(len(shapes)):
        mom[i].copy_(torch.from_numpy(M1[i]))
        w[i].copy_(torch.from_numpy(W1[i]))
        signs[i].zero_()
        counts[i].zero_()
    plan2 = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, sign_fmt=fmt, local_polar_steps=Kp, scale=scale,
                       power_iters=2, v0=v0, signs_out=signs, counts_out=counts)
    P.signmuon_step(ctx, plan2)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        assert np.array_equal(signs[i].cpu().numpy(), g_signs[i]), f"untapped signs block {i}"
        assert np.array_equal(counts[i].cpu().numpy(), g_counts[i]), f"untapped counts block {i}"
        assert np.array_equal(w[i].cpu().numpy().view(np.uint32), g_w[i].view(np.uint32)), f"untapped W block {i}"
    ctx.close()
    del W0


def test_nanogpt124m_step_in_bench_configuration(P):
    # one block of every distinct shape gets the full Newton-Schulz comparison
    full_step_check(P, "nanogpt124m", ns_blocks={0, 1, 2, 3, 47})


@pytest.mark.parametrize("opts", [dict(gemm_tile=128), dict(gemm_tile=256, ns_store="full"),
                                  dict(gemm_tile=256, ns_path="single")],
                         ids=["t128", "t256-full", "t256-single"])
def test_nanogpt124m_step_under_other_settings(P, opts):
    full_step_check(P, "nanogpt124m", ns_blocks={1, 3}, **opts)


def test_resnet50_step_in_bench_configuration(P):
    full_step_check(P, "resnet50", ns_blocks={0, 1, 2, 3, 4, 5})


def test_resnet50_step_with_large_tiles(P):
    full_step_check(P, "resnet50", ns_blocks={3, 5}, gemm_tile=256)


def progress(msg):
    """Progress line of the minute-long tests (visible with pytest -s)."""
    print(msg, flush=True)


def streamed_full_step_check(P, name, ns_items, mom_workers):
    """One step of a large workload from zero momentum, in the benchmark's configuration, checked block by
    block so that the host only ever holds one block.  Bit-exact on ALL blocks and workers: signs, counts
    (hence the vote) and W; momentum bit-exact on all blocks for the workers in mom_workers; Newton-Schulz
    outputs against the float32 oracle on the (block, worker) pairs in ns_items (one per distinct shape) and
    by the rank bound on the rest."""
    import bench
    cfg, w, mom, grad = bench.make_inputs(name, torch, torch.device("cuda:0"))
    shapes, M = cfg["shapes"], cfg["M"]
    K, Kp, fmt = cfg["ns_steps"], cfg["local_polar_steps"], cfg["sign_fmt"]
    lr, beta = 1e-3, 0.9
    d = [r * c for r, c in shapes]
    stride = [O.packed_stride_bytes(x) if fmt == "1bit" else x for x in d]
    w0 = [t.clone() for t in w]
    signs = [torch.zeros((M, s), dtype=torch.uint8, device="cuda") for s in stride]
    counts = [torch.zeros((x,), dtype=torch.int32, device="cuda") for x in d]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    ctx = P.Context()
    plan = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, sign_fmt=fmt, local_polar_steps=Kp,
                      signs_out=signs, counts_out=counts, u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    ns_blocks = {i for i, _ in ns_items}
    ties = 0
    for i, (r, c) in enumerate(shapes):
        progress(f"{name}: checking block {i} of {len(shapes)} ({r} x {c})")
        workers = sorted(set(mom_workers) | {p for bi, p in ns_items if bi == i})
        G = grad[i][workers].cpu().numpy()
        m_ref = O.momentum_update(np.zeros_like(G), G, None, beta, 0.0, dtype=np.float32)
        del G
        assert np.array_equal(mom[i][workers].cpu().numpy().view(np.uint32), m_ref.view(np.uint32)), f"momentum block {i}"
        U = u_out[i].float().cpu().numpy()
        assert np.isfinite(U).all()
        for p in range(M):
            x = U[p].reshape(-1)
            assert float(np.dot(x, x)) <= min(r, c) * 1.02, f"block {i} worker {p}: ||U||_F^2 > rank bound"
        for (bi, p) in ns_items:
            if bi == i:
                ref = O.polar_ns(m_ref[workers.index(p)], K, dtype=np.float32)
                rel, agree = rel_and_agree(U[p], ref)
                report_margins(name, [rel], [agree], f"U block {i} worker {p} vs float32 oracle")
                assert rel <= 2e-2 and agree >= 0.999, f"U block {i} worker {p}: rel {rel:.3e} agree {agree:.5f}"
        del m_ref
        bits_ref = np.stack([O.pack_bits(O.sign_entries(U[p])) for p in range(M)])
        vote_ref, c_ref = O.majority_vote_bits(bits_ref, M, d[i])
        g_signs = signs[i].cpu().numpy()
        if fmt == "1bit":
            assert np.array_equal(g_signs, bits_ref), f"signs block {i}"
        else:
            # +-1 bytes: every byte is +1 or -1 and the +1 pattern is the oracle's bit pattern; the int32 sum
            # is 2 c - M (checked against the int8 oracle itself on the first block)
            s8 = g_signs.view(np.int8)
            assert np.all(np.abs(s8) == 1), f"signs block {i}: byte other than +-1"
            assert np.array_equal(np.stack([O.pack_bits((s8[p] > 0).astype(np.uint8)) for p in range(M)]), bits_ref)
            if i == 0:
                s_ref = np.stack([O.signs_pm1(U[p]).reshape(-1) for p in range(M)])
                assert np.array_equal(s8, s_ref)
                v8, t8 = O.majority_vote_int8(s_ref)
                assert np.array_equal(v8, vote_ref) and np.array_equal(t8, 2 * c_ref - M)
                del s_ref
            c_ref = 2 * c_ref - M
            ties += int(np.sum(c_ref == 0))
        del U, bits_ref, g_signs
        assert np.array_equal(counts[i].cpu().numpy(), c_ref), f"counts block {i}"
        D = d_out[i].float().cpu().numpy()
        S_bar = vote_ref.reshape(r, c)
        if Kp == 0:
            assert np.array_equal(D, S_bar.astype(np.float32))
        else:
            x = D.reshape(-1)
            assert float(np.dot(x, x)) <= min(r, c) * 1.02
            if i in ns_blocks:
                ref = O.local_polar(S_bar, Kp, dtype=np.float32)
                rel, agree = rel_and_agree(D, ref)
                report_margins(name, [rel], [agree], f"D block {i} vs float32 oracle")
                assert rel <= 2e-2 and agree >= 0.999, f"D block {i}: rel {rel:.3e} agree {agree:.5f}"
        w_ref = O.apply_update(w0[i].cpu().numpy(), D, lr, False, dtype=np.float32)
        assert np.array_equal(w[i].cpu().numpy().view(np.uint32), w_ref.view(np.uint32)), f"W block {i}"
    # the benchmark's own configuration has no U tap (the last apply writes only the signs, from its
    # accumulators): same inputs from the same zero state, signs / counts / W equal to the tapped step's
    progress(f"{name}: the same step without the U tap")
    del u_out, d_out, plan
    g_signs = [t.clone() for t in signs]
    g_counts = [t.clone() for t in counts]
    g_w = [t.clone() for t in w]
    for i in range(len(shapes)):
        mom[i].zero_()
        w[i].copy_(w0[i])
        signs[i].zero_()
        counts[i].zero_()
    plan2 = P.StepPlan(w, mom, grad, beta=beta, lr=lr, ns_steps=K, sign_fmt=fmt, local_polar_steps=Kp,
                       signs_out=signs, counts_out=counts)
    P.signmuon_step(ctx, plan2)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        assert torch.equal(signs[i], g_signs[i]), f"untapped signs block {i}"
        assert torch.equal(counts[i], g_counts[i]), f"untapped counts block {i}"
        assert torch.equal(w[i].view(torch.int32), g_w[i].view(torch.int32)), f"untapped W block {i}"
    ctx.close()
    return ties, sum(d)


def test_large_step_in_bench_configuration(P):
    """8 x 4096 x 4096 and 8 x 4096 x 11008, M = 16, Student-t(3) gradients, 1-bit vote, local polar step."""
    streamed_full_step_check(P, "large", ns_items=[(0, 0), (8, 15)], mom_workers=(0, 15))


def test_int8vote_step_in_bench_configuration(P):
    """32 x 2048 x 8192, M = 16, int8 signs summed in int32 (iid workers: about a fifth of the entries tie)."""
    ties, total = streamed_full_step_check(P, "int8vote", ns_items=[(0, 3)], mom_workers=(0, 15))
    assert ties > 0.1 * total


def test_paper_nanogpt_k10_spectral_in_bench_configuration(P):
    """The paper's own nanoGPT shapes (width 384), 10 steps (two segments of the recurrence), spectral scale."""
    full_step_check(P, "nanogpt_paper_k10", ns_blocks={0, 1, 2, 3, 23})


def test_resnet50_k1_spectral_in_bench_configuration(P):
    """One Newton-Schulz step with the spectral scale (the paper's best CIFAR-10 setting)."""
    full_step_check(P, "resnet50_k1", ns_blocks={0, 1, 2, 3, 4, 5})


def test_int8_vote_path_m16_with_ties(P):
    """The int8 transport at M = 16 (iid workers: about a fifth of the entries tie), with a local polar step."""
    shapes, M = [(256, 1024), (1024, 256), (192, 320)], 16
    ctx = P.Context()
    W0 = [wl.weights(r, c, block=i, stream=41) for i, (r, c) in enumerate(shapes)]
    G = [wl.normal((M, r, c), stream=41, block=i) for i, (r, c) in enumerate(shapes)]
    w = [torch.from_numpy(a).cuda() for a in W0]
    mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
    grad = [torch.from_numpy(a).cuda() for a in G]
    d = [r * c for r, c in shapes]
    signs = [torch.zeros((M, x), dtype=torch.int8, device="cuda") for x in d]
    counts = [torch.zeros((x,), dtype=torch.int32, device="cuda") for x in d]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=0.9, lr=1e-2, ns_steps=5, sign_fmt="int8", local_polar_steps=5,
                      signs_out=signs, counts_out=counts, u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    ties = 0
    for i, (r, c) in enumerate(shapes):
        U = u_out[i].float().cpu().numpy()
        s_ref = np.stack([O.signs_pm1(U[p]).reshape(-1) for p in range(M)])
        vote_ref, tot = O.majority_vote_int8(s_ref)
        ties += int(np.sum(tot == 0))
        assert np.array_equal(signs[i].cpu().numpy(), s_ref)
        assert np.array_equal(counts[i].cpu().numpy(), tot)
        D = d_out[i].float().cpu().numpy()
        ref = O.local_polar(vote_ref.reshape(r, c), 5, dtype=np.float32)
        rel, agree = rel_and_agree(D, ref)
        assert rel <= 2e-2 and agree >= 0.999
        w_ref = O.apply_update(W0[i], D, 1e-2, False, dtype=np.float32)
        assert np.array_equal(w[i].cpu().numpy(), w_ref)
    assert ties > 0.1 * sum(d)          # the tie rule really was exercised
    ctx.close()


def test_vector_shaped_and_tiny_blocks(P):
    """Blocks with one dimension equal to 1 (vector parameters treated as m x 1) and a 1 x 1 block."""
    shapes, M = [(1, 96), (96, 1), (1, 1), (3, 5)], 3
    ctx = P.Context()
    W0 = [wl.weights(r, c, block=i, stream=42) for i, (r, c) in enumerate(shapes)]
    G = [wl.normal((M, r, c), stream=42, block=i) for i, (r, c) in enumerate(shapes)]
    w = [torch.from_numpy(a).cuda() for a in W0]
    mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
    grad = [torch.from_numpy(a).cuda() for a in G]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    counts = [torch.zeros((r * c,), dtype=torch.int32, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=0.9, lr=0.5, ns_steps=5, u_out=u_out, counts_out=counts)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    for i, (r, c) in enumerate(shapes):
        m_ref = O.momentum_update(np.zeros_like(G[i]), G[i], None, 0.9, dtype=np.float32)
        U = u_out[i].float().cpu().numpy()
        for p in range(M):
            ref = O.polar_ns(m_ref[p], 5, dtype=np.float32)
            rel, agree = rel_and_agree(U[p], ref)
            assert rel <= 2e-2 and agree >= 0.999, (i, p, rel, agree)
        s_ref = np.stack([O.pack_bits(O.sign_entries(U[p])) for p in range(M)])
        vote, c_ref = O.majority_vote_bits(s_ref, M, r * c)
        assert np.array_equal(counts[i].cpu().numpy(), c_ref)
        assert np.array_equal(w[i].cpu().numpy(), O.apply_update(W0[i], vote.reshape(r, c), 0.5, dtype=np.float32))
    ctx.close()


def test_many_blocks_exceed_one_descriptor_table(P):
    """More blocks than fit one grouped launch (tables hold 40-48 blocks) and more than 32 distinct shapes."""
    shapes = [(64 + 8 * (i % 40), 64) for i in range(70)]
    M = 2
    ctx = P.Context()
    W0 = [wl.weights(r, c, block=i, stream=43) for i, (r, c) in enumerate(shapes)]
    G = [wl.normal((M, r, c), stream=43, block=i) for i, (r, c) in enumerate(shapes)]
    w = [torch.from_numpy(a).cuda() for a in W0]
    mom = [torch.zeros((M, r, c), device="cuda") for r, c in shapes]
    grad = [torch.from_numpy(a).cuda() for a in G]
    u_out = [torch.zeros((M, r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    d_out = [torch.zeros((r, c), dtype=torch.bfloat16, device="cuda") for r, c in shapes]
    plan = P.StepPlan(w, mom, grad, beta=0.9, lr=0.1, ns_steps=3, local_polar_steps=2, u_out=u_out, d_out=d_out)
    P.signmuon_step(ctx, plan)
    torch.cuda.synchronize()
    for i, (r, c) in enumerate(shapes):
        m_ref = O.momentum_update(np.zeros_like(G[i]), G[i], None, 0.9, dtype=np.float32)
        assert np.array_equal(mom[i].cpu().numpy(), m_ref)
        U = u_out[i].float().cpu().numpy()
        ref = O.polar_ns(m_ref[1], 3, dtype=np.float32)
        rel, agree = rel_and_agree(U[1], ref)
        assert rel <= 2e-2 and agree >= 0.999, (i, rel, agree)
        vote = np.where(np.sum(np.where(U >= 0, 1, -1), axis=0) >= 0, 1, -1)
        D = d_out[i].float().cpu().numpy()
        rel, agree = rel_and_agree(D, O.local_polar(vote, 2, dtype=np.float32))
        assert rel <= 2e-2 and agree >= 0.999, (i, rel, agree)
        assert np.array_equal(w[i].cpu().numpy(), O.apply_update(W0[i], D, 0.1, dtype=np.float32))
    ctx.close()
