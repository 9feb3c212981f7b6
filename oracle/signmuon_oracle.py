"""Sign-Muon per-iteration optimizer path: plain CPU oracle.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement
of what the GPU library has to compute.  It shares no code with the HIP path
and must never be imported by the product package; only the tests, the smoke
check and the benchmark's CPU-baseline leg call it.

Every function follows one passage of the Sign-Muon paper ("SignMuon:
Communication-Efficient Distributed Muon Optimization") and says which:

  momentum_update ........ Alg. 1 (single worker) steps 5-6; Alg. 2 steps 6-7
  power_iter ............. Alg. PowerIter (spectral-norm estimate)
  polar_ns ............... Alg. PolarNS; Alg. "Newton-Schulz polar iteration
                           (idealized)" for the free scaling alpha
  sign_entries ........... Alg. 3 note on encoding (>= 0 -> 1, < 0 -> 0)
  pack_bits/unpack_bits .. Alg. 3 step "Pack signs to bits"; appendix
                           "Packed 1-bit representation", eq. (packed-size)
  majority_vote_int8 ..... eq. (mv_def); Alg. 2 "sum_signs" + "ties default
                           to +1"; Lemma "majority vote equals sign of a
                           sum-reduction"
  majority_vote_bits ..... appendix "Majority vote from gathered bits":
                           sum = 2c - M with c the count of +1 bits
  local_polar ............ Sec. "Sign-Muon update" (optional polar(S-bar)
                           after aggregation); appendix "Spectral
                           normalization and polar decomposition are local"
  apply_update ........... Alg. 1 step 9 / Alg. 2 last step; eq.
                           (signmuon_update) for the 1/sqrt(mn) factor
  signmuon_step .......... Alg. 2 / Alg. 3 with the M workers as a leading
                           array dimension

All of it is pinned by tests that do not go through this file's own
formulas (SVD polar factor from LAPACK, per-singular-value closed form,
brute-force votes, the paper's worked payload example); no function here
is "parity unpinned".

Readings taken where the paper leaves a choice (each is stated again at the
function that takes it):
  * sign(0): the algorithms' encoding note wins over the theory's sgn(0)=0:
    bit = (x >= 0) by IEEE comparison, so -0.0 -> 1 and NaN -> 0.
  * vote ties -> +1 (Alg. 2 / Alg. 3).
  * Gram side: the paper always writes Y^T Y (c x c).  For r < c the
    identical map is evaluated with the r x r Gram Y Y^T (same polynomial of
    the singular values); gram="paper" forces the literal form.
  * bit order: entry i of the flattened row-major block is bit (i mod 8) of
    byte (i div 8); a worker's buffer is padded with zero bits to a whole
    number of 64-bit words.
  * int8 signs are summed in a wide integer (the paper's int8 SUM would
    overflow beyond 127 workers).
"""
from __future__ import annotations

import numpy as np

PAPER_COEFFS = (1.5, -0.5, 0.0)  # Y <- 1/2 Y (3I - Y^T Y), Alg. PolarNS


# --------------------------------------------------------------------------
# a1: weight decay + momentum
# --------------------------------------------------------------------------
def momentum_update(mom, grad, w, beta, weight_decay=0.0, dtype=np.float64):
    """G~ = G + lambda W ; M <- beta M + (1 - beta) G~  for every worker.

    mom, grad: [M, r, c]; w: [r, c] (the shared W_t) or None when lambda = 0.
    In the float32 variant every product and sum is rounded on its own
    (no fused multiply-add), and 1 - beta is formed in float32.
    """
    T = np.dtype(dtype).type
    g = np.asarray(grad, dtype=dtype)
    if weight_decay != 0.0:
        g = g + T(weight_decay) * np.asarray(w, dtype=dtype)[None, ...]
    one_minus_beta = T(1.0) - T(beta)
    return T(beta) * np.asarray(mom, dtype=dtype) + one_minus_beta * g


# --------------------------------------------------------------------------
# a2: scale
# --------------------------------------------------------------------------
def power_iter(X, P, eps, v0):
    """Alg. PowerIter.  The paper samples v; here the sample is an input."""
    X = np.asarray(X)
    T = X.dtype.type
    v = np.asarray(v0, dtype=X.dtype)
    v = v / (np.linalg.norm(v) + T(eps))
    for _ in range(int(P)):
        u = X @ v
        u = u / (np.linalg.norm(u) + T(eps))
        v = X.T @ u
        v = v / (np.linalg.norm(v) + T(eps))
    return np.linalg.norm(X @ v)


def scale_sigma(X, scale, power_iters=2, eps=1e-12, v0=None):
    """sigma of Alg. PolarNS: Frobenius norm, PowerIter estimate, or 1."""
    if scale == "fro":
        return np.sqrt(np.sum(np.square(X), dtype=X.dtype))
    if scale == "spectral":
        if v0 is None:
            raise ValueError("spectral scaling needs the start vector v0")
        return power_iter(X, power_iters, eps, v0)
    if scale == "none":
        return X.dtype.type(1.0)
    raise ValueError(f"unknown scale {scale!r}")


# --------------------------------------------------------------------------
# a3 + a4: Newton-Schulz polar iteration
# --------------------------------------------------------------------------
def polar_ns(X, steps, coeffs=PAPER_COEFFS, scale="fro", power_iters=2,
             eps=1e-12, v0=None, dtype=np.float64, gram="short"):
    """Alg. PolarNS on one r x c matrix.

    Y0 = X / max(sigma, eps); then `steps` times
        A = Y^T Y ;  Y <- Y (a I + b A + c A^2)
    which for (a, b, c) = (3/2, -1/2, 0) is the paper's 1/2 Y (3I - Y^T Y).
    gram="short" evaluates the same map through Y Y^T when r < c.
    """
    X = np.asarray(X, dtype=dtype)
    T = X.dtype.type
    r, c = X.shape
    a, b, cc = (T(t) for t in coeffs)
    sigma = scale_sigma(X, scale, power_iters, eps, v0)
    Y = X / max(sigma, T(eps))
    left = (gram == "short") and (r < c)
    if gram not in ("short", "paper"):
        raise ValueError(gram)
    for _ in range(int(steps)):
        if left:
            A = Y @ Y.T
            B = a * np.eye(r, dtype=dtype) + b * A
            if cc != 0:
                B = B + cc * (A @ A)
            Y = B @ Y
        else:
            A = Y.T @ Y
            B = a * np.eye(c, dtype=dtype) + b * A
            if cc != 0:
                B = B + cc * (A @ A)
            Y = Y @ B
    return Y


# --------------------------------------------------------------------------
# a5: sign extraction and packing
# --------------------------------------------------------------------------
def sign_entries(U):
    """Entrywise transmitted sign as a 0/1 array: 1 iff U >= 0 (IEEE compare)."""
    return (np.asarray(U) >= 0).astype(np.uint8)


def signs_pm1(U):
    """The same decision as +1/-1 int8 (the int8 transport of Alg. 2)."""
    return np.where(np.asarray(U) >= 0, 1, -1).astype(np.int8)


def packed_bytes(d):
    """eq. (packed-size): ceil(d / 8) bytes for d sign entries."""
    return -(-int(d) // 8)


def packed_stride_bytes(d):
    """Buffer stride used on the device: whole 64-bit words, >= packed_bytes."""
    return 8 * (-(-int(d) // 64))


def pack_bits(bits01):
    """PackBits: 8 signs per byte, entry i -> bit (i mod 8) of byte (i div 8);
    zero padded to packed_stride_bytes(d).  bits01: flat 0/1 array."""
    bits01 = np.asarray(bits01, dtype=np.uint8).reshape(-1)
    d = bits01.size
    out = np.zeros(packed_stride_bytes(d), dtype=np.uint8)
    out[:packed_bytes(d)] = np.packbits(bits01, bitorder="little")
    return out


def unpack_bits(packed, d):
    """UnpackBits: first d bits, as 0/1."""
    return np.unpackbits(np.asarray(packed, dtype=np.uint8), count=int(d),
                         bitorder="little")


# --------------------------------------------------------------------------
# a6: majority vote
# --------------------------------------------------------------------------
def majority_vote_int8(S):
    """S: [M, d] int8 with entries +-1.  Returns (vote +-1 int8 [d], sum int32 [d]).
    vote = +1 where the integer sum is >= 0 (ties -> +1)."""
    total = np.sum(np.asarray(S, dtype=np.int8).astype(np.int32), axis=0, dtype=np.int32)
    return np.where(total >= 0, 1, -1).astype(np.int8), total


def majority_vote_bits(packed, M, d):
    """packed: [M, stride] uint8 gathered buffers.  Returns
    (vote +-1 int8 [d], c int32 [d]) with c_i the number of +1 bits and
    vote_i = sign(2 c_i - M), ties -> +1."""
    packed = np.asarray(packed, dtype=np.uint8).reshape(int(M), -1)
    c = np.zeros(int(d), dtype=np.int32)
    for p in range(int(M)):
        c += unpack_bits(packed[p], d)
    return np.where(2 * c - int(M) >= 0, 1, -1).astype(np.int8), c


# --------------------------------------------------------------------------
# a7 + a8: local shaping of the voted sign and the parameter update
# --------------------------------------------------------------------------
def local_polar(S_bar, steps, coeffs=PAPER_COEFFS, scale="fro", power_iters=2,
                eps=1e-12, v0=None, dtype=np.float64):
    """D = PolarNS(S-bar; K') when steps > 0, else D = S-bar."""
    S = np.asarray(S_bar, dtype=dtype)
    if steps <= 0:
        return S
    return polar_ns(S, steps, coeffs, scale, power_iters, eps, v0, dtype)


def normalized_sign(S_bar, power_iters, eps, v0, dtype=np.float64):
    """The "normalized sign" direction D = S-bar / ||S-bar||_op of the appendix "Spectral
    normalization and polar decomposition are local", with the operator norm estimated by
    Alg. PowerIter from the start vector v0: D = kappa S-bar, kappa = 1 / max(sigma, eps)."""
    T = np.dtype(dtype).type
    S = np.asarray(S_bar, dtype=dtype)
    sigma = power_iter(S, power_iters, eps, np.asarray(v0, dtype=dtype))
    kappa = T(1.0) / max(T(sigma), T(eps))
    return kappa * S


def apply_update(W, D, lr, rsqrt_mn=False, dtype=np.float64):
    """W <- W - eta * kappa * D, kappa = 1/sqrt(mn) if rsqrt_mn else 1.
    The step eta*kappa is formed first (in `dtype`), then one multiply and
    one subtract per entry."""
    T = np.dtype(dtype).type
    W = np.asarray(W, dtype=dtype)
    r, c = W.shape
    step = T(lr)
    if rsqrt_mn:
        step = T(lr) / np.sqrt(T(r) * T(c))
    return W - step * np.asarray(D, dtype=dtype)


# --------------------------------------------------------------------------
# whole path, one weight block, M workers batched
# --------------------------------------------------------------------------
def signmuon_step(W, mom, grad, *, beta, weight_decay=0.0, lr, ns_steps,
                  coeffs=PAPER_COEFFS, scale="fro", power_iters=2, eps=1e-12,
                  v0=None, sign_fmt="1bit", local_polar_steps=0,
                  rsqrt_mn=False, op_norm=False, dtype=np.float64):
    """One Sign-Muon iteration on one block.  W: [r, c]; mom, grad: [M, r, c];
    v0: [M, c] or None.  Returns dict with the new W and momentum and every
    intermediate (U, packed/int8 signs, counts, vote, D)."""
    M, r, c = np.asarray(grad).shape
    d = r * c
    new_mom = momentum_update(mom, grad, W, beta, weight_decay, dtype)
    U = np.stack([
        polar_ns(new_mom[p], ns_steps, coeffs, scale, power_iters, eps,
                 None if v0 is None else v0[p], dtype)
        for p in range(M)])
    if sign_fmt == "1bit":
        signs = np.stack([pack_bits(sign_entries(U[p])) for p in range(M)])
        vote, counts = majority_vote_bits(signs, M, d)
    elif sign_fmt == "int8":
        signs = np.stack([signs_pm1(U[p]).reshape(-1) for p in range(M)])
        vote, counts = majority_vote_int8(signs)
    else:
        raise ValueError(sign_fmt)
    S_bar = vote.reshape(r, c)
    if op_norm:
        if local_polar_steps > 0 or rsqrt_mn:
            raise ValueError("op_norm shapes the voted sign itself: no local polar step, no 1/sqrt(mn)")
        D = normalized_sign(S_bar, power_iters, eps, v0[0], dtype)
    else:
        D = local_polar(S_bar, local_polar_steps, coeffs, scale, power_iters, eps,
                        None if v0 is None else v0[0], dtype)
    new_W = apply_update(W, D, lr, rsqrt_mn, dtype)
    return dict(W=new_W, mom=new_mom, U=U, signs=signs, counts=counts,
                vote=S_bar, D=D)
