"""Float64 CPU oracle for DeMo's per-step compression path.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
correct numpy implementation of what the HIP kernels must compute, written from
the paper's algorithm statement.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path (the HIP library
and its Python binding) never does, and shares no code with it.

Every function follows the paper's steps in the paper's order, in float64:

  encode (worker side) -- Algorithm 1 "DeMo: Decoupled Momentum", worker loop;
      appendix algorithm "Decoupled Momentum Optimization" (worker side);
      appendix algorithm CompressChunks.
  decode (server side) -- Algorithm 1, parameter-server loop; appendix
      algorithm Decompress&Aggregate; update rule of Sec. 2.1 "Momentum
      Reconstruction and Parameter Update".

Readings taken where the paper is silent or at odds with itself (the full list
with reasons is kept in the design document):

  * momentum update is  m <- beta*m + g  (all four algorithm boxes), not the
    (1-beta)-weighted form of the first display equation of Sec. 2.1;
  * the projection matrix is the textbook orthonormal DCT-II (the paper only
    requires "the DCT", unitary, inverse = transpose);
  * Top-k keeps exactly k coefficients (Sec. 2.1 "Top-k Sparsification",
    ||Q^||_0 = k); equal magnitudes are ordered by lowest flat index first;
  * the flat index of coefficient (u, v) of an s x s chunk is u*s + v with u the
    frequency along tensor dimension 0;
  * the payload of a chunk lists its k pairs by descending magnitude;
  * aggregation is the plain sum over workers (Algorithm 1; Decompress&Aggregate);
  * subtraction coefficient alpha = 1 (algorithm boxes);
  * sgn(0) = 0 (case analysis in the appendix lemma on |x| - x sign(y));
  * the parameter update is evaluated in float32 with two fused multiply-adds,
        t = fma(lambda, x, sgn(m));   x' = fma(-eta, t, x),
    then rounded to the storage type (round-to-nearest-even for bfloat16).  The
    paper does not fix this precision; where a rounding decides the stored code
    both sides must round the same way, so the oracle mimics float32 here.

Variants of the method's scalars and of the server-side aggregate, all off by
default (the defaults are the readings above):

  * grad_scale: coefficient of g in the momentum update; 1 - beta gives the
    weighted form of the first display equation of Sec. 2.1;
  * alpha: coefficient of the subtracted reconstruction (display equation of
    "Momentum Subtraction as Error Feedback"; ablation "Impact of Momentum
    Subtraction", alpha in [0, 1]); the payload still carries the coefficients
    themselves;
  * phi: "sign" (Signum) or "identity" (SGD) in the update rule of "Momentum
    Reconstruction and Parameter Update"; Muon's phi is not covered;
  * aggregate mode: "sum" (algorithm boxes), "mean" (sum / W, the AvgAllGather
    of "Top-k Sparsification") or "count" (appendix algorithm "Sparse Top-k
    Averaging": S (/) n with 0/0 = 0, n = how many workers sent the coefficient);
  * P: any orthonormal s x s matrix in place of the DCT (ablation "Choice of
    Linear Projections": the identity, or Gaussian entries orthonormalised by
    Gram-Schmidt -- `gram_schmidt`, rows in order; drawing the entries is the
    caller's business).

Parity pins (tests/test_oracle_pins.py): DCT against scipy's orthonormal DCT-II,
orthonormality, Parseval, closed forms (constant and single-cosine chunks),
hand-worked 4-point and 4x4 examples, brute-force top-k, k = M exact recovery,
the l1/l2 residual bounds of the appendix lemma and remarks, linearity of the
aggregate, the 128x512 -> 16x32 blocking example, bfloat16 rounding against
torch's conversion, and for the variants: k = M with alpha (residual (1-alpha) m),
alpha = 0, a hand-worked weighted momentum, W identical full payloads under the
mean, the identity update in closed form, and a hand-worked two-worker example of
the count-normalised average; Gram-Schmidt against numpy's QR and a hand-worked
2 x 2 case, the identity basis as plain top-k of the momentum entries.  No
function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "dct_basis", "gram_schmidt", "chunk", "unchunk", "momentum_update", "dct_chunks",
    "idct_chunks", "topk_indices", "encode", "aggregate", "aggregate_counts", "decode", "step",
    "round_to_bf16", "sgn",
]


# --------------------------------------------------------------------------
# Projection matrix  (Sec. 2.1 "Blockwise Linear Projection"; appendix
# "Multilinear Transforms and Chunk-wise Tensor Blocking": unitary, P^T = P^-1)
# --------------------------------------------------------------------------
def dct_basis(s: int) -> np.ndarray:
    """Orthonormal DCT-II matrix  P[u, n] = c_u cos(pi (2n+1) u / (2s)),
    c_0 = sqrt(1/s), c_u = sqrt(2/s) for u > 0."""
    u = np.arange(s, dtype=np.float64)[:, None]
    n = np.arange(s, dtype=np.float64)[None, :]
    P = np.cos(np.pi * (2.0 * n + 1.0) * u / (2.0 * s))
    P *= np.sqrt(2.0 / s)
    P[0, :] = np.sqrt(1.0 / s)
    return P


# --------------------------------------------------------------------------
# Blocking operator B and its inverse (appendix, definition of B_k(X):
# (B_k(X))_j = X[k_0 s_0 + j_0, k_1 s_1 + j_1]; dimensions must divide)
# --------------------------------------------------------------------------
def chunk(x: np.ndarray, s0: int, s1: int | None = None) -> np.ndarray:
    """1-D x of length n -> array [c0, s0];  2-D x -> array [c0, c1, s0, s1]
    with out[k0, k1, j0, j1] = x[k0*s0 + j0, k1*s1 + j1]."""
    if x.ndim == 1:
        if x.shape[0] % s0:
            raise ValueError("length not divisible by chunk size")
        return x.reshape(x.shape[0] // s0, s0).copy()
    if x.ndim != 2:
        raise ValueError("only order-1 and order-2 tensors")
    if s1 is None:
        s1 = s0
    n0, n1 = x.shape
    if n0 % s0 or n1 % s1:
        raise ValueError("shape not divisible by chunk size")
    out = np.empty((n0 // s0, n1 // s1, s0, s1), dtype=x.dtype)
    for k0 in range(n0 // s0):
        for k1 in range(n1 // s1):
            out[k0, k1] = x[k0 * s0:(k0 + 1) * s0, k1 * s1:(k1 + 1) * s1]
    return out


def unchunk(b: np.ndarray) -> np.ndarray:
    """Inverse of `chunk` (concatenation of the blocks)."""
    if b.ndim == 2:
        return b.reshape(-1).copy()
    c0, c1, s0, s1 = b.shape
    x = np.empty((c0 * s0, c1 * s1), dtype=b.dtype)
    for k0 in range(c0):
        for k1 in range(c1):
            x[k0 * s0:(k0 + 1) * s0, k1 * s1:(k1 + 1) * s1] = b[k0, k1]
    return x


def gram_schmidt(A: np.ndarray) -> np.ndarray:
    """Rows of the square matrix A orthonormalised in order by the Gram-Schmidt process (ablation
    "Choice of Linear Projections": Gaussian entries, then Gram-Schmidt; the paper does not say
    rows or columns -- rows are taken, row 0 keeps its direction).  Each row has its projections on
    the rows already finished removed one after the other, then is normalised."""
    A = np.asarray(A, np.float64)
    P = np.zeros_like(A)
    for i in range(A.shape[0]):
        v = A[i].copy()
        for j in range(i):
            v -= np.dot(P[j], v) * P[j]
        P[i] = v / np.sqrt(np.dot(v, v))
    return P


# --------------------------------------------------------------------------
# Step 1: local momentum  (Algorithm 1, "update local momentum buffer")
# --------------------------------------------------------------------------
def momentum_update(m_prev: np.ndarray, g: np.ndarray, beta: float, grad_scale: float = 1.0) -> np.ndarray:
    return (np.float64(beta) * np.asarray(m_prev, np.float64)
            + np.float64(grad_scale) * np.asarray(g, np.float64))


# --------------------------------------------------------------------------
# Step 2: chunk-wise transform T and its inverse
# (d = 2:  Q = P_0 B P_1^T ;  inverse uses the transposed matrices)
# --------------------------------------------------------------------------
def dct_chunks(b: np.ndarray, P: np.ndarray) -> np.ndarray:
    """b: [c0, s] (1-D chunks) or [c0, c1, s, s].  Returns same shape."""
    if b.ndim == 2:
        return b @ P.T                                      # q = P b, per chunk (rows of b)
    return P @ b @ P.T                                      # Q = P B P^T, per chunk


def idct_chunks(q: np.ndarray, P: np.ndarray) -> np.ndarray:
    if q.ndim == 2:
        return q @ P                                        # b = P^T q, per chunk (rows of q)
    return P.T @ q @ P                                      # B = P^T Q P, per chunk


# --------------------------------------------------------------------------
# Step 3: top-k by magnitude inside one chunk, exactly k entries
# --------------------------------------------------------------------------
def topk_indices(q_flat: np.ndarray, k: int) -> np.ndarray:
    """Flat indices of the k largest |q| of one chunk, by descending magnitude;
    equal magnitudes in ascending index order (stable sort)."""
    M = q_flat.shape[0]
    if not 1 <= k <= M:
        raise ValueError("k must satisfy 1 <= k <= M")
    order = np.argsort(-np.abs(q_flat), kind="stable")
    return order[:k].astype(np.int32)


# --------------------------------------------------------------------------
# Worker side, one tensor
# --------------------------------------------------------------------------
def encode(m_prev: np.ndarray, g: np.ndarray, beta: float, s: int, k: int,
           forced_idx: np.ndarray | None = None, alpha: float = 1.0, grad_scale: float = 1.0,
           P: np.ndarray | None = None):
    """One worker's encode of one tensor.

    m_prev, g : float arrays of identical shape ([n] or [n0, n1]); their values
                are used exactly (bfloat16 / float32 inputs are exact in float64).
    forced_idx: optional [nchunks, k] index sets to use instead of the oracle's
                own top-k (the parity tests use it to evaluate values and the
                residual on a selection that differs only inside a near-tie).
    alpha     : coefficient of the subtracted reconstruction (1 = algorithm boxes).
    grad_scale: coefficient of g in the momentum update (1 = algorithm boxes).
    P         : s x s orthonormal projection matrix used for every dimension; default the DCT.
    Returns dict with
      m_new  : residual momentum, same shape as m_prev
      idx    : int32 [nchunks, k]   (chunk order row-major over (k0, k1))
      val    : float64 [nchunks, k] (the coefficients at idx)
      Q      : all coefficients, float64 [nchunks, M]
      m_mid  : beta*m + grad_scale*g before the subtraction
    """
    P = dct_basis(s) if P is None else np.asarray(P, np.float64)
    m_mid = momentum_update(m_prev, g, beta, grad_scale)
    b = chunk(m_mid, s)                                     # ChunkExtract
    Q = dct_chunks(b, P)                                    # DCT
    M = s if m_mid.ndim == 1 else s * s
    nch = b.shape[0] if m_mid.ndim == 1 else b.shape[0] * b.shape[1]
    Qf = Q.reshape(nch, M)
    idx = np.empty((nch, k), np.int32)
    val = np.empty((nch, k), np.float64)
    Qhat = np.zeros_like(Qf)
    for c in range(nch):                                    # Top-k per chunk
        sel = topk_indices(Qf[c], k) if forced_idx is None else np.asarray(forced_idx[c], np.int64)
        idx[c] = sel
        val[c] = Qf[c, sel]
        Qhat[c, sel] = Qf[c, sel]
    resid = b - np.float64(alpha) * idct_chunks(Qhat.reshape(Q.shape), P)   # B <- B - alpha IDCT(q_sp)
    m_new = unchunk(resid).reshape(m_mid.shape)             # ChunkInsert
    return {"m_new": m_new, "idx": idx, "val": val, "Q": Qf, "m_mid": m_mid}


# --------------------------------------------------------------------------
# Server side, one tensor
# --------------------------------------------------------------------------
def aggregate(idx: np.ndarray, val: np.ndarray, M: int) -> np.ndarray:
    """Sum of the sparse coefficients over workers, per chunk.
    idx, val: [W, nchunks, k].  Workers are added in order w = 0..W-1; indices
    outside [0, M) are ignored.  Returns float64 [nchunks, M]."""
    W, nch, k = idx.shape
    S = np.zeros((nch, M), np.float64)
    rows = np.repeat(np.arange(nch), k).reshape(nch, k)
    for w in range(W):                                      # s <- s + Lookup(Q^w, c)
        iw = np.asarray(idx[w], np.int64)
        ok = (iw >= 0) & (iw < M)
        np.add.at(S, (rows[ok], iw[ok]), np.asarray(val[w], np.float64)[ok])
    return S


def aggregate_counts(idx: np.ndarray, M: int) -> np.ndarray:
    """n of the appendix algorithm "Sparse Top-k Averaging": how many workers sent
    each coefficient.  idx: [W, nchunks, k]; returns int64 [nchunks, M]."""
    W, nch, k = idx.shape
    n = np.zeros((nch, M), np.int64)
    rows = np.repeat(np.arange(nch), k).reshape(nch, k)
    for w in range(W):                                      # n_I <- n_I + 1
        iw = np.asarray(idx[w], np.int64)
        ok = (iw >= 0) & (iw < M)
        np.add.at(n, (rows[ok], iw[ok]), 1)
    return n


def sgn(x: np.ndarray) -> np.ndarray:
    return np.sign(x)                                       # sign(0) = 0


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float32
    values that are exactly representable in bfloat16."""
    f = np.asarray(x, np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32)
    nan = np.isnan(f)
    if nan.any():
        out = out.copy()
        out[nan] = np.float32(np.nan)
    return out.reshape(f.shape)


def decode(x: np.ndarray, idx: np.ndarray, val: np.ndarray, lr: float, weight_decay: float,
           s: int, param_dtype: str = "f32", phi: str = "sign", aggregate_mode: str = "sum",
           P: np.ndarray | None = None):
    """Server side for one tensor: aggregate W payloads, inverse transform,
    sign, parameter update.

    x   : parameters ([n] or [n0, n1]), values used exactly
    idx : int [W, nchunks, k];  val: float [W, nchunks, k]
    phi : "sign" or "identity";  aggregate_mode: "sum", "mean" or "count"
    Returns dict with x_new (float32 values, representable in `param_dtype`),
    R (the reconstructed momentum, float64, same shape as x).
    """
    P = dct_basis(s) if P is None else np.asarray(P, np.float64)
    x64 = np.asarray(x, np.float64)
    M = s if x64.ndim == 1 else s * s
    S = aggregate(np.asarray(idx), np.asarray(val, np.float64), M)
    if aggregate_mode == "mean":
        S = S / np.float64(np.asarray(idx).shape[0])
    elif aggregate_mode == "count":
        n = aggregate_counts(np.asarray(idx), M)
        S = np.divide(S, n, out=np.zeros_like(S), where=n > 0)   # S (/) n, 0/0 = 0
    elif aggregate_mode != "sum":
        raise ValueError("aggregate_mode must be 'sum', 'mean' or 'count'")
    if x64.ndim == 1:
        R = unchunk(idct_chunks(S.reshape(-1, s), P))
    else:
        c0, c1 = x64.shape[0] // s, x64.shape[1] // s
        R = unchunk(idct_chunks(S.reshape(c0, c1, s, s), P))
    R = R.reshape(x64.shape)
    if phi == "sign":
        x_new = _sign_update_f32(x64, sgn(R), lr, weight_decay)
    elif phi == "identity":
        x_new = _sign_update_f32(x64, R, lr, weight_decay)   # same two FMAs with phi(m) = m
    else:
        raise ValueError("phi must be 'sign' or 'identity'")
    if param_dtype == "bf16":
        x_new = round_to_bf16(x_new)
    elif param_dtype != "f32":
        raise ValueError("param_dtype must be 'f32' or 'bf16'")
    return {"x_new": x_new, "R": R}


def _fma_f32(a: np.ndarray, b: np.ndarray, c: np.ndarray) -> np.ndarray:
    """float32 fused multiply-add of float32-valued inputs: the product of two
    24-bit significands is exact in float64; one rounding to float32 follows the
    float64 sum (a second rounding only matters on a 2^-29 measure of inputs)."""
    return (np.asarray(a, np.float64) * np.asarray(b, np.float64)
            + np.asarray(c, np.float64)).astype(np.float32)


def _sign_update_f32(x64: np.ndarray, sg: np.ndarray, lr: float, wd: float) -> np.ndarray:
    """x' = x - eta (phi(m) + lambda x)   (Algorithm 1, parameter update line; `sg` is phi(m))."""
    lr32 = np.float32(lr)
    wd32 = np.float32(wd)
    x32 = x64.astype(np.float32)
    t = _fma_f32(wd32, x32, sg.astype(np.float32))
    return _fma_f32(-lr32, t, x32)


def step(m_prev, g, x, beta, lr, weight_decay, s, k, param_dtype="f32", alpha=1.0, grad_scale=1.0,
         phi="sign", aggregate_mode="sum"):
    """encode followed by decode of the worker's own payload (W = 1).  The
    payload carries float32 values, so the decode side sees them rounded."""
    e = encode(m_prev, g, beta, s, k, alpha=alpha, grad_scale=grad_scale)
    payload_val = e["val"].astype(np.float32)
    d = decode(x, e["idx"][None], payload_val[None], lr, weight_decay, s, param_dtype, phi, aggregate_mode)
    return {**e, **d}
