"""Comparators between the HIP path's outputs and the float64 oracle.

Several results are correct when coefficient magnitudes (nearly) tie, so encode
is compared in two stages:
  1. the GPU's index set is legitimate: exactly k distinct in-range indices; with
     thr = the oracle's k-th largest magnitude, every selected coefficient has
     oracle magnitude >= thr*(1 - 1e-6) and every unselected one <= thr*(1 + 1e-6)
     (so the sets are identical unless magnitudes differ by less than 1e-6 relative);
  2. on the GPU's own set, the values and the residual momentum match the oracle's
     within 1e-5 of the chunk's largest magnitude.
Decode: the updated parameters must equal the oracle's bit for bit wherever the
reconstructed momentum is not within rounding noise of zero (|R| > 1e-5 * max|R| of
the chunk); inside that band any of sgn in {-1, 0, +1} is accepted.  Outside the band the
parameters are also held against the update line of Algorithm 1 evaluated in plain float64,
x - eta (sgn(m) + lambda x), rounded once to the storage type: every element within one unit
in the last place (taken at the largest of |x|, |x'| and the step eta |sgn(m) + lambda x|) plus
eta times half a float32 unit of the inner sum, and the number of elements that differ at all is
reported.
"""
from __future__ import annotations

import numpy as np

from oracle import demo_oracle as O

TIE_REL = 1e-6        # relative gap below which two magnitudes count as tied
VAL_REL = 1e-5        # values / momentum: relative to the chunk's max magnitude
SIGN_BAND = 1e-5      # |R| below this fraction of the chunk max: sign is rounding noise


def chunk_rows(x: np.ndarray, s: int) -> np.ndarray:
    """[nchunks, M] view of a tensor in chunk order."""
    b = O.chunk(np.asarray(x), s)
    return b.reshape(-1, s) if x.ndim == 1 else b.reshape(b.shape[0] * b.shape[1], s * s)


def _unchunk_rows(rows: np.ndarray, shape, s: int) -> np.ndarray:
    """Inverse of chunk_rows for an order-2 tensor of `shape`."""
    c0, c1 = shape[0] // s, shape[1] // s
    return O.unchunk(rows.reshape(c0, c1, s, s))


def check_encode(m_prev, g, beta32, s, k, gpu_idx, gpu_val, gpu_m, val_rel=VAL_REL, alpha32=1.0, grad_scale32=1.0,
                 P=None):
    """All arrays numpy; m_prev/g exact input values; gpu_* the HIP outputs.
    Returns a dict of statistics; raises AssertionError on a violation."""
    m_prev = np.asarray(m_prev, np.float64)
    g = np.asarray(g, np.float64)
    var = dict(alpha=float(np.float32(alpha32)), grad_scale=float(np.float32(grad_scale32)), P=P)
    ref = O.encode(m_prev, g, float(np.float32(beta32)), s, k, **var)
    Q = ref["Q"]
    nch, M = Q.shape
    gpu_idx = np.asarray(gpu_idx).reshape(nch, k).astype(np.int64)
    gpu_val = np.asarray(gpu_val, np.float64).reshape(nch, k)
    absQ = np.abs(Q)
    # ---- stage 1: legitimacy of the index sets
    assert gpu_idx.min() >= 0 and gpu_idx.max() < M, "index out of range"
    srt = np.sort(gpu_idx, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1]), "duplicate index inside a chunk"
    thr = np.abs(ref["val"]).min(axis=1)                       # oracle's k-th largest magnitude
    sel_mag = np.take_along_axis(absQ, gpu_idx, 1)
    assert np.all(sel_mag >= thr[:, None] * (1 - TIE_REL)), "selected a coefficient below the threshold"
    mask = np.ones_like(absQ, bool)
    np.put_along_axis(mask, gpu_idx, False, 1)
    unsel_max = np.where(mask, absQ, 0.0).max(axis=1) if k < M else np.zeros(nch)
    assert np.all(unsel_max <= thr * (1 + TIE_REL)), "left out a coefficient above the threshold"
    same = np.array([set(a) == set(b) for a, b in zip(gpu_idx.tolist(), ref["idx"].tolist())])
    # ---- payload order: descending magnitude (GPU's own values), ties by ascending index
    gm = np.abs(gpu_val)
    assert np.all(gm[:, :-1] >= gm[:, 1:]), "payload not sorted by descending magnitude"
    eq = gm[:, :-1] == gm[:, 1:]
    assert np.all(gpu_idx[:, :-1][eq] < gpu_idx[:, 1:][eq]), "equal magnitudes not in ascending index order"
    # ---- stage 2: values and residual on the GPU's own selection
    forced = O.encode(m_prev, g, float(np.float32(beta32)), s, k, forced_idx=gpu_idx, **var)
    scale_q = absQ.max(axis=1)
    err_val = np.abs(gpu_val - forced["val"]).max(axis=1)
    ok = err_val <= val_rel * scale_q
    assert np.all(ok), f"payload values off: worst {np.max(err_val / np.maximum(scale_q, 1e-300)):.3e}"
    ref_m = chunk_rows(forced["m_new"], s)
    got_m = chunk_rows(np.asarray(gpu_m, np.float64), s)
    scale_m = np.abs(chunk_rows(forced["m_mid"], s)).max(axis=1)
    err_m = np.abs(got_m - ref_m).max(axis=1)
    assert np.all(err_m <= val_rel * scale_m), f"momentum off: worst {np.max(err_m / np.maximum(scale_m, 1e-300)):.3e}"
    return {
        "chunks": nch,
        "sets_identical": int(same.sum()),
        "tie_swaps": int((~same).sum()),
        "max_rel_err_val": float(np.max(err_val / np.maximum(scale_q, 1e-300))),
        "max_rel_err_mom": float(np.max(err_m / np.maximum(scale_m, 1e-300))),
    }


def storage_ulp(w: np.ndarray, param_dtype: str) -> np.ndarray:
    """Spacing of the storage type at |w| (8 significant bits for bfloat16, 24 for float32)."""
    return np.exp2(np.floor(np.log2(np.maximum(np.abs(w), 1e-300))) - (7 if param_dtype == "bf16" else 23)) + 1e-45


def round_once(w: np.ndarray, param_dtype: str) -> np.ndarray:
    """float64 values rounded once (nearest, ties to even) to the storage type, returned as float64."""
    if param_dtype != "bf16":
        return w.astype(np.float32).astype(np.float64)
    m, e = np.frexp(w)
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def check_decode(x_prev, idx, val, lr32, wd32, s, param_dtype, gpu_x, phi="sign", aggregate_mode="sum", P=None):
    """x_prev exact parameter values before the call; idx/val the W payloads the GPU consumed.
    phi = "identity": the update is a real number, so the parameters are compared numerically:
    within lr * 1e-5 * (largest |R| of the chunk) plus one unit in the last place of the storage type."""
    x_prev = np.asarray(x_prev, np.float64)
    ref = O.decode(x_prev, np.asarray(idx), np.asarray(val), float(np.float32(lr32)), float(np.float32(wd32)),
                   s, param_dtype, phi, aggregate_mode, P)
    got = np.asarray(gpu_x, np.float32)
    want = ref["x_new"]
    if phi == "identity":
        R = chunk_rows(ref["R"], s)
        tolR = float(np.float32(lr32)) * VAL_REL * np.abs(R).max(axis=1, keepdims=True)
        w = chunk_rows(want.astype(np.float64), s)
        # one unit in the last place: the spacing of the storage type at |w| (8 significant bits for bf16, 24 for f32)
        ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(w), 1e-300))) - (7 if param_dtype == "bf16" else 23)) + 1e-45
        err = np.abs(chunk_rows(got.astype(np.float64), s) - w)
        assert np.all(err <= tolR + ulp), f"parameters off: worst excess {np.max(err - tolR - ulp):.3e}"
        return {"elements": int(got.size), "mismatch": int((got != want).sum()), "in_band": 0,
                "max_err_over_lr_Rmax": float(np.max(err / np.maximum(tolR / VAL_REL, 1e-300)))}
    bad = got != want
    stats = {"elements": int(got.size), "mismatch": int(bad.sum()), "in_band": 0}
    R = chunk_rows(ref["R"], s)
    band = SIGN_BAND * np.abs(R).max(axis=1, keepdims=True)
    in_band = np.abs(R) <= band
    # the update line of Algorithm 1 in plain float64, one rounding to the storage type
    lr64, wd64 = float(np.float32(lr32)), float(np.float32(wd32))
    exact = x_prev - lr64 * (np.sign(ref["R"]) + wd64 * x_prev)
    off = np.abs(got.astype(np.float64) - exact)
    sure = ~in_band.reshape(-1) if x_prev.ndim == 1 else ~_unchunk_rows(in_band, x_prev.shape, s)
    # one unit in the last place at the largest of |x|, |x'| and the step: where x and the step nearly cancel, x' is
    # smaller than the float32 rounding of the step itself
    step = np.abs(lr64 * (np.sign(ref["R"]) + wd64 * x_prev))
    ulp = storage_ulp(np.maximum(np.maximum(np.abs(exact), np.abs(x_prev)), step), param_dtype)
    # ... plus the rounding of the inner sum sgn + lambda x to float32 (half a unit of 2^-23 at magnitude 1), carried
    # through the multiplication by eta: with lambda != 0 and |x'| just above a power of two the two roundings of the
    # float32 evaluation add up to 1.01 units (seen once in 4.7 million elements)
    ulp = ulp + lr64 * 2.0 ** -24 * np.abs(np.sign(ref["R"]) + wd64 * x_prev)
    assert np.all(off[sure] <= ulp[sure]), (
        f"parameters more than one unit in the last place from the float64 update: worst {np.max(off[sure]):.3e}")
    stats["differs_from_f64_update"] = int(np.sum((got.astype(np.float64) != round_once(exact, param_dtype)) & sure))
    if bad.any():
        badc = chunk_rows(bad, s)
        assert not np.any(badc & ~in_band), (
            f"{int(np.sum(badc & ~in_band))} parameters differ where the sign is not in doubt")
        # inside the band the value must still be the update for some sign in {-1, 0, +1}
        alts = []
        for sg in (-1.0, 0.0, 1.0):
            a = O._sign_update_f32(x_prev, np.full_like(x_prev, sg), float(np.float32(lr32)), float(np.float32(wd32)))
            alts.append(O.round_to_bf16(a) if param_dtype == "bf16" else a)
        okalt = (got == alts[0]) | (got == alts[1]) | (got == alts[2])
        assert np.all(okalt[bad]), "in-band parameter is not an update by any sign"
        stats["in_band"] = int(bad.sum())
    return stats
