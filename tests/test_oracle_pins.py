"""Pins of the float64 oracle against facts fixed by the paper and by mathematics
(no GPU, no product code).  Each test names what it would catch."""
import itertools

import numpy as np
import pytest
import scipy.fft
import torch

from oracle import demo_oracle as O


# ---- projection matrix ----------------------------------------------------
@pytest.mark.parametrize("s", [4, 32, 64, 128])
def test_basis_orthonormal(s):
    # appendix "Multilinear Transforms ...": the DCT matrix is unitary, P^T = P^-1
    P = O.dct_basis(s)
    assert np.abs(P @ P.T - np.eye(s)).max() < 1e-13
    assert np.abs(P.T @ P - np.eye(s)).max() < 1e-13


@pytest.mark.parametrize("s", [4, 32, 64, 128])
def test_dct_matches_library_routine(s):
    # the transform reduces to the library's orthonormal DCT-II; catches a wrong
    # normalisation, a wrong phase (2n+1) and a transposed operand (P^T B P)
    rng = np.random.default_rng(s)
    b1 = rng.standard_normal((5, s))
    b2 = rng.standard_normal((2, 3, s, s))
    P = O.dct_basis(s)
    assert np.allclose(O.dct_chunks(b1, P), scipy.fft.dct(b1, type=2, norm="ortho", axis=-1), atol=1e-12)
    assert np.allclose(O.dct_chunks(b2, P), scipy.fft.dctn(b2, type=2, norm="ortho", axes=(-2, -1)), atol=1e-12)
    assert np.allclose(O.idct_chunks(b1, P), scipy.fft.idct(b1, type=2, norm="ortho", axis=-1), atol=1e-12)
    assert np.allclose(O.idct_chunks(b2, P), scipy.fft.idctn(b2, type=2, norm="ortho", axes=(-2, -1)), atol=1e-12)


def test_dct_closed_forms():
    s = 64
    P = O.dct_basis(s)
    # constant chunk c -> only the DC coefficient: c*s (2-D), c*sqrt(s) (1-D)
    q2 = O.dct_chunks(np.full((1, 1, s, s), 0.25), P)[0, 0]
    assert abs(q2[0, 0] - 0.25 * s) < 1e-12 and np.abs(q2).sum() - abs(q2[0, 0]) < 1e-10
    q1 = O.dct_chunks(np.full((1, s), 0.25), P)[0]
    assert abs(q1[0] - 0.25 * np.sqrt(s)) < 1e-12 and np.abs(q1[1:]).max() < 1e-12
    # a separable cosine  cos(pi(2i+1)u/2s) cos(pi(2j+1)v/2s)  -> a single coefficient at (u, v),
    # u along dimension 0: catches swapped frequency axes
    u, v = 3, 10
    i = np.arange(s)
    blk = np.outer(np.cos(np.pi * (2 * i + 1) * u / (2 * s)), np.cos(np.pi * (2 * i + 1) * v / (2 * s)))
    Q = O.dct_chunks(blk[None, None], P)[0, 0]
    assert abs(Q[u, v] - s / 2) < 1e-10
    Q[u, v] = 0
    assert np.abs(Q).max() < 1e-10


def test_parseval():
    rng = np.random.default_rng(1)
    for s in (32, 64):
        P = O.dct_basis(s)
        b = rng.standard_normal((2, 2, s, s))
        Q = O.dct_chunks(b, P)
        assert np.allclose((Q ** 2).sum((-1, -2)), (b ** 2).sum((-1, -2)), rtol=1e-12)


# ---- blocking operator ------------------------------------------------------
def test_blocking_example_128x512():
    # appendix "Example (Matrix Blocking)": 128 x 512 into 16 x 32 blocks,
    # (B_{k0,k1})_{j0,j1} = X[16 k0 + j0, 32 k1 + j1], k0 in [0,8), k1 in [0,16)
    X = np.arange(128 * 512, dtype=np.float64).reshape(128, 512)
    B = O.chunk(X, 16, 32)
    assert B.shape == (8, 16, 16, 32)
    for k0, k1, j0, j1 in [(0, 0, 0, 0), (0, 0, 15, 31), (7, 15, 15, 31), (3, 9, 4, 17), (1, 0, 0, 5)]:
        assert B[k0, k1, j0, j1] == X[16 * k0 + j0, 32 * k1 + j1]
    assert np.array_equal(O.unchunk(B), X)
    with pytest.raises(ValueError):
        O.chunk(X, 24, 32)


# ---- hand-worked examples ---------------------------------------------------
def test_hand_example_1d(golden):
    G = golden("hand_1d_s4.txt")
    e = O.encode(np.array(G["m_prev"]), np.array(G["g"]), G["beta"][0], 4, 2)
    assert np.allclose(e["m_mid"], G["m_mid"], atol=1e-15)
    assert np.allclose(e["Q"][0], G["q"], atol=1e-13)
    assert e["idx"][0].tolist() == [int(v) for v in G["idx"]]
    assert np.allclose(e["val"][0], [G["q"][0], G["q"][1]], atol=1e-13)
    assert np.allclose(e["m_new"], G["m_new"], atol=1e-13)
    # decode of the own payload reproduces IDCT(q_hat); all positive -> x <- x - lr
    x = np.array([0.5, -0.25, 0.0, 1.0])
    d = O.decode(x, e["idx"][None], e["val"][None], 2.0 ** -10, 0.0, 4)
    assert np.allclose(d["R"], G["idct_qhat"], atol=1e-13)
    assert np.array_equal(d["x_new"], (x - 2.0 ** -10).astype(np.float32))
    # near tie (equal in exact arithmetic): either completion is legitimate
    t = O.encode(np.zeros(4), np.array(G["tie_m_mid"]), 0.9, 4, 2)
    assert np.allclose(t["Q"][0], G["tie_q"], atol=1e-13)
    assert t["idx"][0, 0] == int(G["tie_idx_first"][0])
    assert t["idx"][0, 1] in [int(v) for v in G["tie_idx_second_any_of"]]
    # exact tie (all-zero chunk): lowest flat indices first, zero values, momentum untouched
    z = O.encode(np.zeros(8), np.zeros(8), 0.9, 4, 2)
    assert z["idx"].tolist() == [[0, 1], [0, 1]] and not z["val"].any() and not z["m_new"].any()


def test_hand_example_2d(golden):
    G = golden("hand_2d_s4.txt")
    B = np.array(G["B"]).reshape(4, 4)
    e = O.encode(np.zeros((4, 4)), B, 0.999, 4, 3)
    Q = e["Q"][0].reshape(4, 4)
    assert np.allclose(Q[0], G["Q_row0"], atol=1e-12)
    assert np.allclose(Q[:, 0], G["Q_col0"], atol=1e-12)
    assert np.abs(Q[1:, 1:]).max() < 1e-12
    assert e["idx"][0].tolist() == [int(v) for v in G["idx"]]
    assert np.allclose(e["m_new"][0], G["resid_row0"], atol=1e-12)
    assert np.allclose(e["m_new"][1], G["resid_row1"], atol=1e-12)
    assert np.allclose(e["m_new"][::-1, ::-1], -e["m_new"], atol=1e-12)


# ---- top-k --------------------------------------------------------------------
def test_topk_brute_force():
    # all k on tiny chunks, with repeated magnitudes: compare with an explicit
    # search over all k-subsets for the maximal (magnitude desc, index asc) choice
    rng = np.random.default_rng(7)
    for trial in range(40):
        q = rng.integers(-3, 4, size=6).astype(np.float64)        # many ties
        for k in range(1, 7):
            got = O.topk_indices(q, k).tolist()
            assert len(set(got)) == k
            best = max(itertools.combinations(range(6), k),
                       key=lambda c: (sum(abs(q[i]) for i in c), [-i for i in c]))
            thr = min(abs(q[i]) for i in got)
            assert all(abs(q[i]) <= thr for i in range(6) if i not in got)
            assert sum(abs(q[i]) for i in got) == sum(abs(q[i]) for i in best)
            # ties resolved towards the lowest index, output by descending magnitude
            keyed = sorted(range(6), key=lambda i: (-abs(q[i]), i))[:k]
            assert got == keyed


def test_topk_domain():
    with pytest.raises(ValueError):
        O.topk_indices(np.ones(4), 0)
    with pytest.raises(ValueError):
        O.topk_indices(np.ones(4), 5)


# ---- encode invariants ------------------------------------------------------
@pytest.mark.parametrize("shape,s", [((128,), 32), ((64, 128), 32), ((128, 64), 64)])
def test_k_equals_M_exact_recovery(shape, s):
    # appendix remark on isometric transformations: k = M gives perfect reconstruction,
    # so the residual momentum is zero and decode of the own payload returns m_mid
    rng = np.random.default_rng(3)
    m, g = rng.standard_normal(shape), rng.standard_normal(shape)
    M = s if len(shape) == 1 else s * s
    e = O.encode(m, g, 0.999, s, M)
    assert np.abs(e["m_new"]).max() < 1e-12
    assert sorted(e["idx"][0].tolist()) == list(range(M))
    d = O.decode(np.zeros(shape), e["idx"][None], e["val"][None], 1e-3, 0.0, s)
    assert np.allclose(d["R"], e["m_mid"], atol=1e-12)


@pytest.mark.parametrize("k", [1, 8, 32])
def test_residual_bounds_and_split(k):
    rng = np.random.default_rng(11)
    s = 32
    m, g = rng.standard_normal((64, 96)) * 1e-3, rng.standard_normal((64, 96)) * 1e-2
    e = O.encode(m, g, 0.999, s, k)
    M = s * s
    P = O.dct_basis(s)
    Q = e["Q"]
    Qhat = np.zeros_like(Q)
    np.put_along_axis(Qhat, e["idx"].astype(np.int64), e["val"], axis=1)
    # lemma "Optimal Universal l1-norm Bound": ||X* - X||_1 <= (1 - k/M) ||X||_1
    assert np.all(np.abs(Q - Qhat).sum(1) <= (1 - k / M) * np.abs(Q).sum(1) + 1e-15)
    # l2 remark through the isometry, per chunk, plus the exact Pythagoras split
    b_mid = O.chunk(e["m_mid"], s).reshape(-1, M)
    b_new = O.chunk(e["m_new"], s).reshape(-1, M)
    n_mid, n_new = (b_mid ** 2).sum(1), (b_new ** 2).sum(1)
    assert np.all(np.sqrt(n_new) <= np.sqrt(1 - k / M) * np.sqrt(n_mid) + 1e-15)
    assert np.allclose(n_mid, (e["val"] ** 2).sum(1) + n_new, rtol=1e-11)
    # the DCT of the residual vanishes at the selected slots and is below the threshold elsewhere
    Qres = O.dct_chunks(O.chunk(e["m_new"], s), P).reshape(-1, M)
    thr = np.abs(e["val"]).min(1)
    assert np.abs(np.take_along_axis(Qres, e["idx"].astype(np.int64), 1)).max() < 1e-14
    assert np.all(np.abs(Qres).max(1) <= thr + 1e-15)
    # payload size: nchunks*k pairs, reduction M/k  (Sec. 2.1 "Top-k Sparsification")
    assert e["idx"].shape == (6, k) and e["val"].shape == (6, k)


def test_momentum_update_form():
    # Algorithm 1: m <- beta m + g (gradient unweighted)
    e = O.encode(np.full(4, 2.0), np.full(4, 1.0), 0.5, 4, 4)
    assert np.array_equal(e["m_mid"], np.full(4, 2.0))


def test_forced_indices():
    rng = np.random.default_rng(5)
    g = rng.standard_normal((32, 32))
    e0 = O.encode(np.zeros((32, 32)), g, 0.9, 32, 4)
    alt = e0["idx"].copy()
    alt[0, 3] = (int(alt[0, 0]) + 1) % 1024 if (int(alt[0, 0]) + 1) % 1024 not in alt[0] else 1023
    e1 = O.encode(np.zeros((32, 32)), g, 0.9, 32, 4, forced_idx=alt)
    assert np.array_equal(e1["val"][0], e0["Q"][0, alt[0]])


# ---- decode -------------------------------------------------------------------
def test_aggregate_is_ordered_sum_and_linear():
    rng = np.random.default_rng(2)
    W, nch, k, s = 5, 4, 6, 8
    idx = np.stack([np.stack([rng.permutation(s * s)[:k] for _ in range(nch)]) for _ in range(W)]).astype(np.int32)
    idx[1] = idx[0]                                     # forced collisions between workers
    val = rng.standard_normal((W, nch, k))
    S = O.aggregate(idx, val, s * s)
    ref = np.zeros((nch, s * s))
    for w in range(W):
        for c in range(nch):
            for t in range(k):
                ref[c, idx[w, c, t]] += val[w, c, t]
    assert np.array_equal(S, ref)
    # linearity (Sec. 2.1): decoding W payloads = sum of the single-payload reconstructions,
    # and mean instead of sum leaves every sign unchanged
    x = np.zeros((16, 16))
    d_all = O.decode(x, idx, val, 1e-3, 0.0, s)
    parts = sum(O.decode(x, idx[w:w + 1], val[w:w + 1], 1e-3, 0.0, s)["R"] for w in range(W))
    assert np.allclose(d_all["R"], parts, atol=1e-13)
    d_mean = O.decode(x, idx, val / W, 1e-3, 0.0, s)
    assert np.array_equal(np.sign(d_mean["R"]), np.sign(d_all["R"]))
    # out-of-range indices are ignored
    bad = idx.copy()
    bad[0, 0, 0] = s * s
    bad[0, 0, 1] = -1
    S2 = O.aggregate(bad, val, s * s)
    fix = val.copy()
    fix[0, 0, :2] = 0.0
    assert np.allclose(S2, O.aggregate(idx, fix, s * s))


def test_sign_update_closed_form():
    s = 4
    P = O.dct_basis(s)
    # one DC coefficient -> constant positive block; one negative; one empty (sgn 0 = 0)
    idx = np.zeros((1, 3, 1), np.int32)
    val = np.array([[[2.0], [-3.0], [0.0]]])
    x = np.linspace(-1, 1, 12)
    d = O.decode(x, idx, val, 0.125, 0.0, s)
    assert np.array_equal(np.sign(d["R"]), np.repeat([1.0, -1.0, 0.0], 4))
    assert np.allclose(d["x_new"], x - 0.125 * np.repeat([1.0, -1.0, 0.0], 4), atol=1e-7)
    # weight decay: x' = x - eta (sgn + lambda x); empty chunk only shrinks x
    d = O.decode(x, idx, val, 0.125, 0.5, s)
    expect = x - 0.125 * (np.repeat([1.0, -1.0, 0.0], 4) + 0.5 * x)
    assert np.allclose(d["x_new"], expect, atol=1e-7)
    # 2-D placement: coefficient (u=1, v=0) varies along dimension 0 only
    idx2 = np.full((1, 1, 1), 1 * s + 0, np.int32)
    d2 = O.decode(np.zeros((4, 4)), idx2, np.ones((1, 1, 1)), 1.0, 0.0, s)
    assert np.allclose(d2["R"], np.outer(P[1], P[0]), atol=1e-14)
    assert np.array_equal(d2["x_new"], -np.sign(np.outer(P[1], P[0])).astype(np.float32))


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 0.02,
                        np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -1.001953125, 0.0, 3.0e38])])
    x = x.astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_to_bf16(x), ref)
    # exact half-way cases go to the even neighbour
    assert O.round_to_bf16(np.float32(1.00390625)) == np.float32(1.0)          # 1 + 2^-8 -> 1
    assert O.round_to_bf16(np.float32(1.01171875)) == np.float32(1.015625)     # 1 + 3*2^-8 -> 1 + 2^-6


def test_bf16_param_update():
    # lr = 1e-3 from -0.5 towards -0.501: below half a bfloat16 ulp (2^-9), rounded away;
    # from +0.5 downwards the ulp is 2^-9 and the step survives; small |x| moves.  Values are those of float32 arithmetic followed by one RNE rounding.
    x = O.round_to_bf16(np.array([0.5, -0.5, 0.01, -0.01, 0.0], np.float32)).astype(np.float64)
    idx = np.zeros((1, 5, 1), np.int32)
    val = np.ones((1, 5, 1))
    d = O.decode(np.repeat(x, 4), idx, val, 1e-3, 0.0, 4, "bf16")["x_new"].reshape(5, 4)[:, 0]
    ref = (torch.tensor(x, dtype=torch.float32) - torch.tensor(1e-3, dtype=torch.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(d, ref)
    assert d[1] == np.float32(-0.5) and d[0] == np.float32(0.5 - 2.0 ** -9) and d[2] < np.float32(0.01)


def test_step_is_encode_then_decode():
    rng = np.random.default_rng(9)
    m, g, x = rng.standard_normal((32, 64)), rng.standard_normal((32, 64)), rng.standard_normal((32, 64))
    st = O.step(m, g, x, 0.999, 1e-3, 0.1, 32, 8)
    e = O.encode(m, g, 0.999, 32, 8)
    d = O.decode(x, e["idx"][None], e["val"].astype(np.float32)[None], 1e-3, 0.1, 32)
    assert np.array_equal(st["m_new"], e["m_new"]) and np.array_equal(st["x_new"], d["x_new"])


# ---------------------------------------------------------------------------
# Variants of the scalars and of the aggregate (off by default)
# ---------------------------------------------------------------------------
def test_alpha_full_selection_leaves_one_minus_alpha():
    # k = M: the reconstruction is the momentum itself, so the momentum-subtraction equation
    # (Sec. 2.1, "Momentum Subtraction as Error Feedback") leaves (1 - alpha) * (beta m + g)
    rng = np.random.default_rng(21)
    m, g = rng.standard_normal((16, 24)), rng.standard_normal((16, 24))
    for alpha in (0.0, 0.2, 0.5, 1.0):
        e = O.encode(m, g, 0.9, 8, 64, alpha=alpha)
        assert np.allclose(e["m_new"], (1.0 - alpha) * (0.9 * m + g), atol=1e-12)
    v, gv = rng.standard_normal(32), rng.standard_normal(32)
    e = O.encode(v, gv, 0.5, 8, 8, alpha=0.2)
    assert np.allclose(e["m_new"], 0.8 * (0.5 * v + gv), atol=1e-12)


def test_alpha_zero_subtracts_nothing_and_payload_is_unscaled():
    rng = np.random.default_rng(22)
    m, g = rng.standard_normal((16, 16)), rng.standard_normal((16, 16))
    e0 = O.encode(m, g, 0.9, 8, 3, alpha=0.0)
    e1 = O.encode(m, g, 0.9, 8, 3)
    e2 = O.encode(m, g, 0.9, 8, 3, alpha=0.2)
    assert np.array_equal(e0["m_new"], 0.9 * m + g)
    # the transmitted coefficients do not depend on alpha; the residual interpolates linearly
    assert np.array_equal(e0["idx"], e1["idx"]) and np.array_equal(e0["val"], e1["val"])
    assert np.array_equal(e2["val"], e1["val"])
    assert np.allclose(e2["m_new"], 0.8 * e1["m_mid"] + 0.2 * e1["m_new"], atol=1e-12)


def test_weighted_momentum_hand_example():
    # first display equation of Sec. 2.1: M = beta M + (1 - beta) G, worked by hand with beta = 1/2
    m = np.array([2.0, 4.0, 6.0, 8.0])
    g = np.array([4.0, 0.0, -2.0, 2.0])
    e = O.encode(m, g, 0.5, 4, 4, grad_scale=0.5)
    assert np.array_equal(e["m_mid"], np.array([3.0, 2.0, 2.0, 5.0]))
    # k = M = 4 and alpha = 1: everything is sent, nothing is left
    assert np.allclose(e["m_new"], 0.0, atol=1e-14)
    # the DC coefficient of the orthonormal DCT-II of [3, 2, 2, 5] is 12 / sqrt(4) = 6
    dc = e["val"][0][list(e["idx"][0]).index(0)]
    assert abs(dc - 6.0) < 1e-12


def test_identity_phi_and_mean_closed_form():
    # W workers all send every coefficient of the same momentum m: the mean is m's transform, the
    # reconstruction is m, and the SGD form of the update rule gives x - lr (m + wd x) (Sec. 2.1,
    # "Momentum Reconstruction and Parameter Update" with phi = identity)
    rng = np.random.default_rng(23)
    m = rng.standard_normal((16, 16))
    x = rng.standard_normal((16, 16)).astype(np.float32).astype(np.float64)
    e = O.encode(np.zeros_like(m), m, 0.0, 8, 64)
    W = 5
    idx = np.repeat(e["idx"][None], W, 0)
    val = np.repeat(e["val"][None], W, 0)
    d = O.decode(x, idx, val, 0.25, 0.5, 8, phi="identity", aggregate_mode="mean")
    assert np.allclose(d["R"], m, atol=1e-12)
    assert np.allclose(d["x_new"], x - 0.25 * (m + 0.5 * x), rtol=0, atol=2e-6)
    dsum = O.decode(x, idx, val, 0.25, 0.5, 8, phi="identity", aggregate_mode="sum")
    assert np.allclose(dsum["R"], W * m, atol=1e-11)
    # every worker sent every coefficient: the count-normalised average equals the mean
    dcnt = O.decode(x, idx, val, 0.25, 0.5, 8, phi="identity", aggregate_mode="count")
    assert np.allclose(dcnt["R"], m, atol=1e-12)
    # sign descent does not see a positive rescaling of the aggregate
    a = O.decode(x, idx, val, 0.25, 0.5, 8, aggregate_mode="mean")["x_new"]
    b = O.decode(x, idx, val, 0.25, 0.5, 8, aggregate_mode="sum")["x_new"]
    assert np.array_equal(a, b)


def test_count_normalised_average_hand_example():
    # appendix algorithm "Sparse Top-k Averaging", N = 2, d = 4, k = 2, worked by hand:
    #   X1 = [3, -1, 0.5, 2] sends {0: 3, 3: 2};  X2 = [1, 4, -0.2, 3] sends {1: 4, 3: 3}
    #   S = [3, 4, 0, 5], n = [1, 1, 0, 2]  ->  S (/) n = [3, 4, 0, 2.5]  (0/0 = 0)
    X1, X2 = np.array([3.0, -1.0, 0.5, 2.0]), np.array([1.0, 4.0, -0.2, 3.0])
    i1, i2 = O.topk_indices(X1, 2), O.topk_indices(X2, 2)
    assert sorted(i1) == [0, 3] and sorted(i2) == [1, 3]
    idx = np.stack([i1, i2])[:, None, :]
    val = np.stack([X1[i1], X2[i2]])[:, None, :]
    assert np.array_equal(O.aggregate(idx, val, 4), np.array([[3.0, 4.0, 0.0, 5.0]]))
    assert np.array_equal(O.aggregate_counts(idx, 4), np.array([[1, 1, 0, 2]]))
    d = O.decode(np.zeros(4), idx, val, 1.0, 0.0, 4, phi="identity", aggregate_mode="count")
    # the reconstruction's transform (scipy's orthonormal DCT-II, an independent routine) is the average
    assert np.allclose(scipy.fft.dct(d["R"], norm="ortho"), np.array([3.0, 4.0, 0.0, 2.5]), atol=1e-12)
    # not sign-equivalent to the plain sum in general: here coefficient 3 halves
    dsum = O.decode(np.zeros(4), idx, val, 1.0, 0.0, 4, phi="identity", aggregate_mode="sum")
    assert np.allclose(scipy.fft.dct(dsum["R"], norm="ortho"), np.array([3.0, 4.0, 0.0, 5.0]), atol=1e-12)


# ---------------------------------------------------------------------------
# Other projection matrices (ablation "Choice of Linear Projections")
# ---------------------------------------------------------------------------
def test_gram_schmidt_hand_and_qr():
    # hand-worked: rows (3, 4) and (1, 0): first row / 5; second minus its projection 0.6 * (0.6, 0.8)
    # = (0.64, -0.48), of norm 0.8 -> (0.8, -0.6)
    P = O.gram_schmidt(np.array([[3.0, 4.0], [1.0, 0.0]]))
    assert np.allclose(P, np.array([[0.6, 0.8], [0.8, -0.6]]), atol=1e-15)
    rng = np.random.default_rng(40)
    for s in (4, 32, 64, 128):
        A = rng.standard_normal((s, s))
        P = O.gram_schmidt(A)
        assert np.allclose(P @ P.T, np.eye(s), atol=1e-10)
        # Gram-Schmidt on the rows of A is the QR factorisation of A^T with positive diagonal of R
        Qm, Rm = np.linalg.qr(A.T)
        Qm = Qm * np.sign(np.diag(Rm))[None, :]
        assert np.allclose(P, Qm.T, atol=1e-9)
        # row i stays inside the span of the first i + 1 rows of A, along +A[i] modulo earlier rows
        assert np.all(np.diag(P @ A.T) > 0)


def test_identity_basis_is_plain_topk_of_entries():
    rng = np.random.default_rng(41)
    m, g = rng.standard_normal((8, 12)), rng.standard_normal((8, 12))
    e = O.encode(m, g, 0.5, 4, 3, P=np.eye(4))
    mid = 0.5 * m + g
    blocks = O.chunk(mid, 4).reshape(-1, 16)
    for c in range(blocks.shape[0]):
        order = sorted(range(16), key=lambda i: (-abs(blocks[c, i]), i))[:3]
        assert list(e["idx"][c]) == order
        assert np.array_equal(e["val"][c], blocks[c, order])
    # the kept entries are removed, everything else stays
    left = O.chunk(e["m_new"], 4).reshape(-1, 16)
    for c in range(blocks.shape[0]):
        keep = np.ones(16, bool)
        keep[e["idx"][c]] = False
        assert np.array_equal(left[c, keep], blocks[c, keep]) and np.all(left[c, ~keep] == 0.0)


def test_random_orthonormal_basis_exact_recovery_and_parseval():
    rng = np.random.default_rng(42)
    s = 8
    P = O.gram_schmidt(rng.standard_normal((s, s)))
    m = rng.standard_normal((16, 24))
    e = O.encode(np.zeros_like(m), m, 0.0, s, s * s, P=P)
    assert np.allclose(e["m_new"], 0.0, atol=1e-12)
    assert np.allclose((e["Q"] ** 2).sum(), (m ** 2).sum(), rtol=1e-12)
    x = rng.standard_normal((16, 24))
    d = O.decode(x, e["idx"][None], e["val"][None], 0.5, 0.0, s, phi="identity", P=P)
    assert np.allclose(d["R"], m, atol=1e-12)
    # 1-D
    v = rng.standard_normal(32)
    e1 = O.encode(np.zeros(32), v, 0.0, s, s, P=P)
    d1 = O.decode(np.zeros(32), e1["idx"][None], e1["val"][None], 1.0, 0.0, s, phi="identity", P=P)
    assert np.allclose(d1["R"], v, atol=1e-12) and np.allclose(e1["m_new"], 0.0, atol=1e-12)


# ---- bit-level pins of the float32 update epilogue  t = fma(lambda, x, phi),  x' = fma(-eta, t, x) ---------------
def _round_fraction_to_f32(fr):
    """Exact rational -> nearest float32 (ties to even), by integer arithmetic only."""
    from fractions import Fraction
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    fr = abs(Fraction(fr))
    e = 0
    while fr >= 2:
        fr /= 2
        e += 1
    while fr < 1:
        fr *= 2
        e -= 1
    scaled = fr * (1 << 23)                       # significand in [2^23, 2^24)
    q, r = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * r
    if twice > scaled.denominator or (twice == scaled.denominator and (q & 1)):
        q += 1
    return np.float32(sign * float(q) * 2.0 ** (e - 23))


def test_update_epilogue_bits_with_weight_decay():
    upd = lambda x, sg, lr, wd: O._sign_update_f32(np.array([x], np.float64), np.array([sg], np.float64), lr, wd)[0]
    # exact cases: 1 - 0.25 (1 + 0.5*1) = 0.625 ;  -2 - 0.5 (-1 + 0.25*(-2)) = -1.25
    assert upd(1.0, 1.0, 0.25, 0.5) == np.float32(0.625)
    assert upd(-2.0, -1.0, 0.5, 0.25) == np.float32(-1.25)
    # first product-sum lands half-way between two float32 values: 1 + 2^-24 -> 1 (even), then 1 - 0.5 = 0.5
    assert upd(1.0, 1.0, 0.5, 2.0 ** -24) == np.float32(0.5)
    # 1 + 3*2^-24 is half-way between 1 + 2^-23 (odd) and 1 + 2^-22 (even) -> 1 + 2^-22;
    # then 3 - 0.5 (1 + 2^-22) = 2.5 - 2^-23, half-way between 2.5 - 2^-22 and 2.5 (even) -> 2.5
    assert upd(3.0, 1.0, 0.5, 2.0 ** -24) == np.float32(2.5)
    # just above the half-way point the sum rounds up: 1 + 2^-24 + 2^-47 (x = 1 + 2^-23 exactly representable)
    # -> 1 + 2^-23, and x' = x - t = 0 (rounded down to 1 it would leave 2^-23)
    assert upd(1.0 + 2.0 ** -23, 1.0, 1.0, 2.0 ** -24) == np.float32(0.0)
    # the products are not rounded on their own (fused): 1 - fl32(1e-3) * 1, one rounding of the exact difference
    lr32 = float(np.float32(1e-3))
    assert upd(1.0, 1.0, 1e-3, 0.0) == _round_fraction_to_f32(1 - __import__("fractions").Fraction(lr32))
    assert upd(1.0, 1.0, 1e-3, 0.0) == np.float32(16760439.0 * 2.0 ** -24)   # exact difference: 16760438.783... * 2^-24
    # random float32 inputs against exact rational arithmetic with one rounding per fused operation
    from fractions import Fraction
    rng = np.random.default_rng(5)
    for _ in range(400):
        x = float(np.float32(rng.standard_normal() * 0.02))
        sg = float(rng.integers(-1, 2))
        lr, wd = float(np.float32(10.0 ** rng.uniform(-4, -1))), float(np.float32(10.0 ** rng.uniform(-3, 0)))
        t = _round_fraction_to_f32(Fraction(wd) * Fraction(x) + Fraction(sg))
        want = _round_fraction_to_f32(-Fraction(lr) * Fraction(float(t)) + Fraction(x))
        assert upd(x, sg, lr, wd) == want
