"""Pins for the fp64 CPU oracle: everything here checks oracle/ against something
other than itself -- exact rational brute force, library-matmul closed forms,
algebraic invariants and exact finite differences.  No GPU needed.

Passages pinned (Symbiosis, arXiv 2507.03220): Sec. 3.2 (batch, execute, split per
client), Sec. 3.7 (padding-free flattening), Sec. 3.6 (backward = output gradient
times frozen parameters; forward and backward batches are independent), Sec. 3.8
eqs. (1)-(3) (noise linearity with a bias-free pass), Sec. 4 "output exactly
identical to the baseline" (batched == alone).
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth
from helpers import bits_of, f64, grid_bits, tiny_problem

EXACT = dict(rtol=0, atol=0)


# ---------------------------------------------------------------------------
# P1: exact rational brute force, loop nest ordered differently from the C code
# ---------------------------------------------------------------------------
def _frac(bits):
    return [[Fraction(float(v)) for v in row] for row in np.atleast_2d(f64(bits))]


def _brute(p):
    """Every output as an exact Fraction, straight from the per-element definition."""
    off, d_in, d_out = p["off"], p["d_in"], p["d_out"]
    X, W, dY = _frac(p["X"]), _frac(p["W"]), _frac(p["dY"])
    b = [Fraction(float(v)) for v in f64(p["bias"])] if p["bias"] is not None else [Fraction(0)] * d_out
    Y0 = [[None] * d_out for _ in range(p["T"])]
    Y = [[None] * d_out for _ in range(p["T"])]
    dX = [[None] * d_in for _ in range(p["T"])]
    dXb = [[None] * d_in for _ in range(p["T"])]
    grads = {}
    for i, a in enumerate(p["ads"]):
        lo, hi = int(off[i]), int(off[i + 1])
        A = _frac(a.A) if a.A is not None else None
        B = _frac(a.B) if a.B is not None else None
        s = Fraction(a.scale)
        for t in range(lo, hi):
            for j in range(d_out):
                Y0[t][j] = b[j] + sum(W[j][k] * X[t][k] for k in reversed(range(d_in)))
            for k in range(d_in):
                dXb[t][k] = sum(W[j][k] * dY[t][j] for j in reversed(range(d_out)))
        if a.kind == oracle.NONE:
            for t in range(lo, hi):
                Y[t] = list(Y0[t])
                dX[t] = list(dXb[t])
        elif a.kind == oracle.LORA:
            r = a.rank
            dA = [[Fraction(0)] * d_in for _ in range(r)]
            dB = [[Fraction(0)] * r for _ in range(d_out)]
            for t in range(lo, hi):
                H = [sum(X[t][k] * A[q][k] for k in range(d_in)) for q in range(r)]
                dH = [s * sum(dY[t][j] * B[j][q] for j in range(d_out)) for q in range(r)]
                for j in range(d_out):
                    Y[t][j] = Y0[t][j] + s * sum(H[q] * B[j][q] for q in range(r))
                    for q in range(r):
                        dB[j][q] += s * H[q] * dY[t][j]
                for k in range(d_in):
                    dX[t][k] = dXb[t][k] + sum(dH[q] * A[q][k] for q in range(r))
                    for q in range(r):
                        dA[q][k] += X[t][k] * dH[q]
            grads[i] = (dA, dB)
        elif a.kind == oracle.IA3:
            l = A[0]
            dl = [Fraction(0)] * d_out
            for t in range(lo, hi):
                for j in range(d_out):
                    Y[t][j] = l[j] * Y0[t][j]
                    dl[j] += dY[t][j] * Y0[t][j]
                for k in range(d_in):
                    dX[t][k] = sum(dY[t][j] * l[j] * W[j][k] for j in range(d_out))
            grads[i] = dl
        elif a.kind == oracle.IA3_IN:
            l = A[0]
            dl = [Fraction(0)] * d_in
            for t in range(lo, hi):
                for j in range(d_out):
                    Y[t][j] = b[j] + sum(l[k] * X[t][k] * W[j][k] for k in range(d_in))
                for k in range(d_in):
                    dX[t][k] = l[k] * dXb[t][k]
                    dl[k] += X[t][k] * dXb[t][k]
            grads[i] = dl
    tof = lambda M: np.array([[float(v) for v in row] for row in M], dtype=np.float64)
    return tof(Y0), tof(Y), tof(dX), tof(dXb), grads


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("bias", [True, False])
def test_brute_force_exact(seed, bias):
    p = tiny_problem(seed=seed, bias=bias)
    Y0r, Yr, dXr, dXbr, gr = _brute(p)
    Y0, Y = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    np.testing.assert_allclose(Y0, Y0r, **EXACT)
    np.testing.assert_allclose(Y, Yr, **EXACT)
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    np.testing.assert_allclose(dX, dXr, **EXACT)
    dXb = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"], base_only=True)
    np.testing.assert_allclose(dXb, dXbr, **EXACT)
    for i, a in enumerate(p["ads"]):
        if a.kind == oracle.LORA:
            dA, dB = oracle.lora_grad(p["off"], p["ads"], p["X"], p["dY"], i)
            np.testing.assert_allclose(dA, np.array([[float(v) for v in r] for r in gr[i][0]]), **EXACT)
            np.testing.assert_allclose(dB, np.array([[float(v) for v in r] for r in gr[i][1]]), **EXACT)
            if p["off"][i + 1] == p["off"][i]:
                assert not dA.any() and not dB.any()
        elif a.kind in (oracle.IA3, oracle.IA3_IN):
            dl = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], i)
            np.testing.assert_allclose(dl, np.array([float(v) for v in gr[i]]), **EXACT)


def test_row_subset_matches_full():
    p = tiny_problem(seed=5)
    rows = np.array([10, 0, 3, 4, 7], dtype=np.int32)  # unordered, skips the empty segment
    Y0, Y = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    Y0s, Ys = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"], rows=rows)
    np.testing.assert_array_equal(Ys, Y[rows])
    np.testing.assert_array_equal(Y0s, Y0[rows])
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    dXs = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"], rows=rows)
    np.testing.assert_array_equal(dXs, dX[rows])
    dl = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], 2)
    dls = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], 2, cols=[2, 0])
    np.testing.assert_array_equal(dls, dl[[2, 0]])


# ---------------------------------------------------------------------------
# P3: merged-weight closed form through a library fp64 matmul
# ---------------------------------------------------------------------------
def _merged_weight(a, W):
    Wd = f64(W)
    if a.kind == oracle.LORA:
        return Wd + a.scale * (f64(a.B) @ f64(a.A))      # [d_out, r] @ [r, d_in]
    if a.kind == oracle.IA3:
        return f64(a.A)[:, None] * Wd
    if a.kind == oracle.IA3_IN:
        return Wd * f64(a.A)[None, :]
    return Wd


def _random_problem(seed, d_in=48, d_out=40, lens=(9, 1, 0, 17, 5, 30), bias=True):
    rng = np.random.default_rng(seed)
    kinds = [oracle.LORA, oracle.IA3, oracle.LORA, oracle.NONE, oracle.IA3_IN, oracle.LORA]
    ranks = [4, 0, 7, 0, 0, 16]
    off = np.zeros(len(lens) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    T = int(off[-1])
    nb = lambda shape, std, mean=0.0: synth.f32_to_bf16_bits(
        (mean + std * rng.standard_normal(shape)).astype(np.float32))
    ads = []
    for i, k in enumerate(kinds):
        if k == oracle.LORA:
            ads.append(oracle.Adapter(k, ranks[i], 16.0 / ranks[i], nb((ranks[i], d_in), d_in ** -0.5),
                                      nb((d_out, ranks[i]), ranks[i] ** -0.5)))
        elif k == oracle.IA3:
            ads.append(oracle.Adapter(k, 0, 0.0, nb((d_out,), 0.1, 1.0)))
        elif k == oracle.IA3_IN:
            ads.append(oracle.Adapter(k, 0, 0.0, nb((d_in,), 0.1, 1.0)))
        else:
            ads.append(oracle.Adapter())
    return dict(off=off, X=nb((T, d_in), 1.0), W=nb((d_out, d_in), d_in ** -0.5), dY=nb((T, d_out), 1.0),
                bias=nb((d_out,), 0.5) if bias else None, ads=ads, d_in=d_in, d_out=d_out, T=T,
                S=len(lens))


@pytest.mark.parametrize("seed", [3, 4])
def test_merged_weight_closed_form(seed):
    p = _random_problem(seed)
    Y0, Y = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    dXb = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"], base_only=True)
    Xd, dYd, bd = f64(p["X"]), f64(p["dY"]), f64(p["bias"])
    np.testing.assert_allclose(Y0, Xd @ f64(p["W"]).T + bd, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dXb, dYd @ f64(p["W"]), rtol=1e-12, atol=1e-12)
    for i, a in enumerate(p["ads"]):
        lo, hi = p["off"][i], p["off"][i + 1]
        Wm = _merged_weight(a, p["W"])
        bm = bd * f64(a.A) if a.kind == oracle.IA3 else bd   # output scaling scales the bias too
        np.testing.assert_allclose(Y[lo:hi], Xd[lo:hi] @ Wm.T + bm, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(dX[lo:hi], dYd[lo:hi] @ Wm, rtol=1e-12, atol=1e-12)
        # Textbook dense-layer weight gradient of the merged layer, projected on the factors.
        dWm = dYd[lo:hi].T @ Xd[lo:hi]                    # [d_out, d_in]
        if a.kind == oracle.LORA:
            dA, dB = oracle.lora_grad(p["off"], p["ads"], p["X"], p["dY"], i)
            np.testing.assert_allclose(dA, a.scale * f64(a.B).T @ dWm, rtol=1e-11, atol=1e-11)
            np.testing.assert_allclose(dB, a.scale * dWm @ f64(a.A).T, rtol=1e-11, atol=1e-11)
        elif a.kind == oracle.IA3:
            dl = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], i)
            ref = np.sum(dWm * f64(p["W"]), axis=1) + bd * dYd[lo:hi].sum(axis=0)
            np.testing.assert_allclose(dl, ref, rtol=1e-11, atol=1e-11)
        elif a.kind == oracle.IA3_IN:
            dl = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], i)
            np.testing.assert_allclose(dl, np.sum(dWm * f64(p["W"]), axis=0), rtol=1e-11, atol=1e-11)


# ---------------------------------------------------------------------------
# P2: B = 0 and l = 1 reduce to the plain frozen layer
# ---------------------------------------------------------------------------
def test_zero_B_and_unit_l_reduce_to_base():
    p = _random_problem(7)
    for a in p["ads"]:
        if a.kind == oracle.LORA:
            a.B = np.zeros_like(a.B)
        elif a.kind in (oracle.IA3, oracle.IA3_IN):
            a.A = bits_of(np.ones(a.A.shape))
    Y0, Y = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    np.testing.assert_array_equal(Y, Y0)
    np.testing.assert_allclose(Y, f64(p["X"]) @ f64(p["W"]).T + f64(p["bias"]), rtol=1e-12, atol=1e-12)
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    np.testing.assert_array_equal(dX, oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"], base_only=True))
    for i, a in enumerate(p["ads"]):
        if a.kind == oracle.LORA:
            dA, dB = oracle.lora_grad(p["off"], p["ads"], p["X"], p["dY"], i)
            assert not dA.any()                 # dH = s dY B = 0
            if p["off"][i + 1] > p["off"][i]:
                assert dB.any()                 # the B gradient does not vanish with B


# ---------------------------------------------------------------------------
# P4 / P5 / P8: permutation invariance, batched == alone, backward on a sub-batch
# ---------------------------------------------------------------------------
def _sub_batch(p, order):
    """Re-flatten the listed segments, in the listed order, as a batch of its own."""
    off = p["off"]
    idx = np.concatenate([np.arange(off[i], off[i + 1]) for i in order]).astype(np.int64) \
        if len(order) else np.zeros(0, dtype=np.int64)
    noff = np.zeros(len(order) + 1, dtype=np.int32)
    noff[1:] = np.cumsum([off[i + 1] - off[i] for i in order])
    return noff, [p["ads"][i] for i in order], np.ascontiguousarray(p["X"][idx]), \
        np.ascontiguousarray(p["dY"][idx])


@pytest.mark.parametrize("order", [[5, 0, 3, 1, 4, 2], [3], [0], [5, 4], [4, 1, 0]])
def test_segment_regrouping_is_bit_identical(order):
    p = _random_problem(11)
    Y0, Y = oracle.forward(p["off"], p["ads"], p["X"], p["W"], p["bias"])
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    noff, nads, nX, ndY = _sub_batch(p, order)
    _, Yn = oracle.forward(noff, nads, nX, p["W"], p["bias"])
    dXn = oracle.backward_input(noff, nads, ndY, p["W"])
    for q, i in enumerate(order):
        lo, hi = p["off"][i], p["off"][i + 1]
        np.testing.assert_array_equal(Yn[noff[q]:noff[q + 1]], Y[lo:hi])
        np.testing.assert_array_equal(dXn[noff[q]:noff[q + 1]], dX[lo:hi])
        a = p["ads"][i]
        if a.kind == oracle.LORA:
            g0 = oracle.lora_grad(p["off"], p["ads"], p["X"], p["dY"], i)
            g1 = oracle.lora_grad(noff, nads, nX, ndY, q)
            np.testing.assert_array_equal(g0[0], g1[0])
            np.testing.assert_array_equal(g0[1], g1[1])
        elif a.kind in (oracle.IA3, oracle.IA3_IN):
            g0 = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], i)
            g1 = oracle.ia3_grad(noff, nads, nX, ndY, p["W"], p["bias"], q)
            np.testing.assert_array_equal(g0, g1)


# ---------------------------------------------------------------------------
# P6: central finite differences of L = <dY, Y>.  L is linear in X and in each
# adapter tensor separately, and all values sit on an exact grid, so the
# difference quotient is the exact derivative.
# ---------------------------------------------------------------------------
def _loss(p, X=None, ads=None):
    _, Y = oracle.forward(p["off"], ads or p["ads"], p["X"] if X is None else X, p["W"], p["bias"])
    return float(np.sum(Y * f64(p["dY"])))


def _bump(bits, idx, delta):
    v = synth.bf16_bits_to_f32(bits).copy()
    v[idx] += np.float32(delta)
    return bits_of(v)


@pytest.mark.parametrize("seed", [0, 9])
def test_finite_differences_exact(seed):
    p = tiny_problem(seed=seed)
    delta = 0.5
    dX = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"])
    for t in range(p["T"]):
        for k in range(p["d_in"]):
            fd = (_loss(p, X=_bump(p["X"], (t, k), delta)) - _loss(p, X=_bump(p["X"], (t, k), -delta))) / (2 * delta)
            assert fd == dX[t, k], (t, k)
    # base_only differs from the full gradient exactly on adapted, non-empty segments
    dXb = oracle.backward_input(p["off"], p["ads"], p["dY"], p["W"], base_only=True)
    assert not np.array_equal(dXb, dX)

    def with_adapter(i, **kw):
        ads = list(p["ads"])
        a = ads[i]
        ads[i] = oracle.Adapter(a.kind, a.rank, a.scale, kw.get("A", a.A), kw.get("B", a.B))
        return ads

    for i, a in enumerate(p["ads"]):
        if a.kind == oracle.LORA:
            dA, dB = oracle.lora_grad(p["off"], p["ads"], p["X"], p["dY"], i)
            for idx in np.ndindex(*a.A.shape):
                fd = (_loss(p, ads=with_adapter(i, A=_bump(a.A, idx, delta)))
                      - _loss(p, ads=with_adapter(i, A=_bump(a.A, idx, -delta)))) / (2 * delta)
                assert fd == dA[idx], ("dA", i, idx)
            for idx in np.ndindex(*a.B.shape):
                fd = (_loss(p, ads=with_adapter(i, B=_bump(a.B, idx, delta)))
                      - _loss(p, ads=with_adapter(i, B=_bump(a.B, idx, -delta)))) / (2 * delta)
                assert fd == dB[idx], ("dB", i, idx)
        elif a.kind in (oracle.IA3, oracle.IA3_IN):
            dl = oracle.ia3_grad(p["off"], p["ads"], p["X"], p["dY"], p["W"], p["bias"], i)
            for c in range(a.A.shape[0]):
                fd = (_loss(p, ads=with_adapter(i, A=_bump(a.A, (c,), delta)))
                      - _loss(p, ads=with_adapter(i, A=_bump(a.A, (c,), -delta)))) / (2 * delta)
                assert fd == dl[c], ("dl", i, c)


# ---------------------------------------------------------------------------
# P7: noise linearity (Sec. 3.8): fwd(x+n, b) - fwd_nobias(n) == fwd(x, b)
# ---------------------------------------------------------------------------
def test_noise_effect_subtraction_is_exact():
    rng = np.random.default_rng(21)
    d_in, d_out, T = 6, 4, 9
    off = np.array([0, 4, 9], dtype=np.int32)
    ads = [oracle.Adapter(), oracle.Adapter()]
    X, N = grid_bits(rng, (T, d_in), -6, 6), grid_bits(rng, (T, d_in), -6, 6)
    W, b = grid_bits(rng, (d_out, d_in)), grid_bits(rng, (d_out,))
    XN = bits_of(synth.bf16_bits_to_f32(X) + synth.bf16_bits_to_f32(N))
    _, y = oracle.forward(off, ads, X, W, b)
    _, y_noisy = oracle.forward(off, ads, XN, W, b)
    _, n_eff = oracle.forward(off, ads, N, W, None)
    np.testing.assert_array_equal(y_noisy - n_eff, y)


def _round_to_bf16_by_definition(v: Fraction) -> Fraction:
    """Nearest value with an 8-bit significand, ties to the even significand (normal range)."""
    if v == 0:
        return Fraction(0)
    a, e = abs(v), 0
    while a >= 2 ** (e + 1):
        e += 1
    while a < 2 ** e:
        e -= 1
    q = Fraction(2) ** (e - 7)                  # spacing of 8-bit significands in [2^e, 2^(e+1))
    k = a / q
    lo = k.numerator // k.denominator
    r = k - lo
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return (q * lo) * (1 if v > 0 else -1)


def test_noise_add_rounds_the_exact_sum_once():
    """Client prepass x + n (Sec. 3.8): against the exact rational sum rounded by the definition of
    round-to-nearest-even; broadcast, per-token and absent noise, one empty segment."""
    rng = np.random.default_rng(33)
    d = 7
    off = np.array([0, 3, 3, 8, 10], dtype=np.int32)
    X = synth.f32_to_bf16_bits(rng.standard_normal((10, d)).astype(np.float32))
    per_tok = synth.f32_to_bf16_bits(rng.standard_normal((3, d)).astype(np.float32))
    bcast = synth.f32_to_bf16_bits(rng.standard_normal((1, d)).astype(np.float32))
    noise = [per_tok, None, bcast, None]
    out = oracle.noise_add(off, X, noise)
    xf, of = synth.bf16_bits_to_f64(X), synth.bf16_bits_to_f64(out)
    for t in range(10):
        seg = int(np.searchsorted(off, t, side="right") - 1)
        for k in range(d):
            if noise[seg] is None:
                assert out[t, k] == X[t, k]
                continue
            n = synth.bf16_bits_to_f64(noise[seg])[0 if noise[seg].shape[0] == 1 else t - off[seg], k]
            want = _round_to_bf16_by_definition(Fraction(float(xf[t, k])) + Fraction(float(n)))
            assert Fraction(float(of[t, k])) == want, (t, k)
    with pytest.raises(ValueError):
        oracle.noise_add(off, X, [np.zeros((2, d), np.uint16), None, None, None])   # 2 rows for a 3-token segment


def test_private_forward_equals_plain_forward_for_every_adapter_kind():
    """Eqs. (1)-(3) of Sec. 3.8 with adapters on: the layer plus a LoRA / IA3 adapter is still linear, so
    noise added before and its bias-free effect removed after leave the plain result, exactly when
    x + n needs no rounding.  A noise effect computed with the bias in would fail this."""
    p = tiny_problem(seed=5, d_in=6, d_out=4, lens=(3, 0, 2, 2, 4))
    rng = np.random.default_rng(5)
    off, ads = p["off"], p["ads"]
    X = grid_bits(rng, (p["T"], 6), -6, 6)
    noise = [grid_bits(rng, (3, 6), -6, 6), None, grid_bits(rng, (1, 6), -6, 6), None, grid_bits(rng, (4, 6), -6, 6)]
    Xn = oracle.noise_add(off, X, noise)
    # on this grid the sums are exact: Xn holds x + n itself
    full = np.zeros((p["T"], 6))
    for i, n in enumerate(noise):
        if n is not None:
            full[off[i]:off[i + 1]] = f64(n) if n.shape[0] > 1 else np.repeat(f64(n), off[i + 1] - off[i], axis=0)
    np.testing.assert_array_equal(f64(Xn), f64(X) + full)
    _, y = oracle.forward(off, ads, X, p["W"], p["bias"])
    yp = oracle.forward_private(off, ads, Xn, p["W"], p["bias"], noise)
    np.testing.assert_allclose(yp, y, rtol=0, atol=1e-11)
    # rows subset
    rows = np.array([10, 0, 5], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_private(off, ads, Xn, p["W"], p["bias"], noise, rows=rows), yp[rows])


def test_denoise_with_a_stored_noise_effect():
    """Steps (2)-(3) of Sec. 3.8 with the noise effect given as the 16-bit tensor the client kept:
    (a) against an exact rational evaluation written out here (own loop order; per-token, broadcast
    and absent noise effects, an empty segment, IA3 scaling the bias too, a row subset);
    (b) when the stored tensor holds the exact effect of the noise, the result is the plain layer
    output and agrees with the route that recomputes the effect."""
    rng = np.random.default_rng(44)
    d_in, d_out = 6, 4
    off = np.array([0, 3, 3, 5, 9], dtype=np.int32)
    l = grid_bits(rng, (d_out,), 4, 12)
    ads = [oracle.Adapter(), oracle.Adapter(), oracle.Adapter(oracle.IA3, 0, 0.0, l), oracle.Adapter()]
    Xn = grid_bits(rng, (9, d_in), -6, 6)
    W, b = grid_bits(rng, (d_out, d_in), -4, 4), grid_bits(rng, (d_out,))
    neff = [synth.f32_to_bf16_bits(rng.standard_normal((3, d_out)).astype(np.float32)), None,
            synth.f32_to_bf16_bits(rng.standard_normal((1, d_out)).astype(np.float32)), None]
    got = oracle.forward_denoise(off, ads, Xn, W, b, neff)
    F = lambda bits: [[Fraction(float(v)) for v in row] for row in np.atleast_2d(f64(bits))]
    xf, wf, bf_, lf = F(Xn), F(W), F(b)[0], F(l)[0]
    for j in range(d_out):
        for t in range(9):
            seg = 0 if t < 3 else 2 if t < 5 else 3
            y = bf_[j]
            for k in range(d_in):
                y += wf[j][k] * xf[t][k]
            if seg == 2:
                y *= lf[j]
            if neff[seg] is not None:
                y -= F(neff[seg])[0 if neff[seg].shape[0] == 1 else t - int(off[seg])][j]
            assert Fraction(float(got[t, j])) == y, (t, j)
    rows = np.array([8, 0, 4], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_denoise(off, ads, Xn, W, b, neff, rows=rows), got[rows])
    with pytest.raises(ValueError):
        oracle.forward_denoise(off, ads, Xn, W, b, [np.zeros((2, d_out), np.uint16), None, None, None])
    # (b) small grids: n W^T is exactly representable in bf16, so storing it loses nothing
    X = grid_bits(rng, (9, d_in), -3, 3)
    noise = [grid_bits(rng, (3, d_in), -3, 3), None, grid_bits(rng, (1, d_in), -3, 3), None]
    Xn2 = oracle.noise_add(off, X, noise)
    stored = []
    for i, n in enumerate(noise):
        if n is None:
            stored.append(None)
            continue
        noff = np.array([0, n.shape[0]], dtype=np.int32)
        _, e = oracle.forward(noff, [ads[i]], n, W, None)
        stored.append(bits_of(e))                      # asserts exact representability
    _, y = oracle.forward(off, ads, X, W, b)
    yd = oracle.forward_denoise(off, ads, Xn2, W, b, stored)
    np.testing.assert_array_equal(yd, y)
    np.testing.assert_array_equal(yd, oracle.forward_private(off, ads, Xn2, W, b, noise))


# ---------------------------------------------------------------------------
# P9: adapter-index probe with exactly representable values
# ---------------------------------------------------------------------------
def test_client_scaled_tensor_is_the_exact_product_rounded_once():
    """The product an IA3 client forms in 16 bits before the tensor goes to the executor (Sec. 3.2, Sec. 4):
    each element against the exact rational product rounded by the definition of round-to-nearest-even;
    rows of other segments untouched; both kinds."""
    rng = np.random.default_rng(44)
    width = 9
    off = np.array([0, 3, 3, 8, 10], dtype=np.int32)
    V = synth.f32_to_bf16_bits(rng.standard_normal((10, width)).astype(np.float32))
    lvec = lambda: synth.f32_to_bf16_bits((1.0 + 0.3 * rng.standard_normal(width)).astype(np.float32))
    for kind, other in ((oracle.IA3, oracle.IA3_IN), (oracle.IA3_IN, oracle.IA3)):
        ads = [oracle.Adapter(kind, 0, 0.0, lvec()), oracle.Adapter(kind, 0, 0.0, lvec()),
               oracle.Adapter(other, 0, 0.0, lvec()), oracle.Adapter(kind, 0, 0.0, lvec())]
        out = oracle.client_scale(off, ads, V, kind)
        vf, of = f64(V), f64(out)
        n_rounded = 0
        for t in range(10):
            seg = int(np.searchsorted(off, t, side="right") - 1)
            for c in range(width):
                if ads[seg].kind != kind:
                    assert out[t, c] == V[t, c]
                    continue
                exact = Fraction(float(vf[t, c])) * Fraction(float(f64(ads[seg].A)[c]))
                want = _round_to_bf16_by_definition(exact)
                assert Fraction(float(of[t, c])) == want, (kind, t, c)
                n_rounded += want != exact
        assert n_rounded > 20          # the case does exercise the rounding
    with pytest.raises(ValueError):
        oracle.client_scale(off, ads, V, oracle.LORA)


def test_client_route_is_the_plain_layer_on_the_client_scaled_tensor():
    """backward_input / forward with client_bf16: (a) with scale vectors that are powers of two no product
    needs rounding, and the route gives the exact definition bit for bit; (b) in general it is the exact
    definition evaluated on the rounded product, so it differs from the exact result by at most the
    rounding bound 2^-8 sum |term| per element (half a spacing of 8-bit significands is at most 2^-8 of the value), and does differ; (c) base-only calls and batches without
    such segments are untouched."""
    p = tiny_problem(seed=8, d_in=6, d_out=5, lens=(3, 0, 2, 2, 4))       # kinds: LoRA, LoRA, IA3, NONE, IA3_IN
    rng = np.random.default_rng(8)
    off, ads = p["off"], list(p["ads"])
    X = synth.f32_to_bf16_bits(rng.standard_normal((p["T"], 6)).astype(np.float32))
    dY = synth.f32_to_bf16_bits(rng.standard_normal((p["T"], 5)).astype(np.float32))
    W = synth.f32_to_bf16_bits(rng.standard_normal((5, 6)).astype(np.float32))
    b = synth.f32_to_bf16_bits(rng.standard_normal(5).astype(np.float32))
    pow2 = lambda n: bits_of(np.float32(2.0) ** rng.integers(-3, 4, n).astype(np.float32) * rng.choice([-1.0, 1.0], n).astype(np.float32))
    ads_p2 = list(ads)
    ads_p2[2] = oracle.Adapter(oracle.IA3, 0, 0.0, pow2(5))
    ads_p2[4] = oracle.Adapter(oracle.IA3_IN, 0, 0.0, pow2(6))
    np.testing.assert_array_equal(oracle.backward_input(off, ads_p2, dY, W, client_bf16=True), oracle.backward_input(off, ads_p2, dY, W))
    for got, want in zip(oracle.forward(off, ads_p2, X, W, b, client_bf16=True), oracle.forward(off, ads_p2, X, W, b)):
        np.testing.assert_array_equal(got, want)
    # general vectors: within the rounding bound of the exact result, and not equal to it
    ads_g = list(ads)
    ads_g[2] = oracle.Adapter(oracle.IA3, 0, 0.0, synth.f32_to_bf16_bits((1 + 0.3 * rng.standard_normal(5)).astype(np.float32)))
    ads_g[4] = oracle.Adapter(oracle.IA3_IN, 0, 0.0, synth.f32_to_bf16_bits((1 + 0.3 * rng.standard_normal(6)).astype(np.float32)))
    dXe, dXc = oracle.backward_input(off, ads_g, dY, W), oracle.backward_input(off, ads_g, dY, W, client_bf16=True)
    rows3 = slice(off[2], off[3])
    bound = 2.0 ** -8 * (np.abs(f64(dY)[rows3] * f64(ads_g[2].A)) @ np.abs(f64(W)))
    assert (np.abs(dXc - dXe)[rows3] <= bound + 1e-15).all() and np.abs(dXc - dXe)[rows3].max() > 0
    keep = np.ones(p["T"], bool); keep[rows3] = False
    np.testing.assert_array_equal(dXc[keep], dXe[keep])
    (Y0e, Ye), (Y0c, Yc) = oracle.forward(off, ads_g, X, W, b), oracle.forward(off, ads_g, X, W, b, client_bf16=True)
    rows5 = slice(off[4], off[5])
    bound = 2.0 ** -8 * (np.abs(f64(X)[rows5] * f64(ads_g[4].A)) @ np.abs(f64(W)).T)
    assert (np.abs(Yc - Ye)[rows5] <= bound + 1e-15).all() and np.abs(Yc - Ye)[rows5].max() > 0
    keep = np.ones(p["T"], bool); keep[rows5] = False
    np.testing.assert_array_equal(Yc[keep], Ye[keep])
    np.testing.assert_array_equal(Y0c, Y0e)
    # row subsets go through the same route
    rows = np.array([off[3] - 1, 0, off[5] - 1], dtype=np.int32)
    np.testing.assert_array_equal(oracle.backward_input(off, ads_g, dY, W, rows=rows, client_bf16=True), dXc[rows])
    np.testing.assert_array_equal(oracle.forward(off, ads_g, X, W, b, rows=rows, client_bf16=True)[1], Yc[rows])
    # untouched: base-only, and a batch with no such segment
    np.testing.assert_array_equal(oracle.backward_input(off, ads_g, dY, W, base_only=True, client_bf16=True),
                                  oracle.backward_input(off, ads_g, dY, W, base_only=True))
    plain = [a if a.kind == oracle.LORA else oracle.Adapter() for a in ads_g]
    np.testing.assert_array_equal(oracle.backward_input(off, plain, dY, W, client_bf16=True), oracle.backward_input(off, plain, dY, W))


def test_index_probe_recovers_row_to_adapter_map():
    lens = [3, 0, 1, 5, 1, 1, 0, 7, 2]
    S = len(lens)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(lens)
    T, d_in, d_out = int(off[-1]), 4, 6
    Xf = np.zeros((T, d_in), np.float32); Xf[:, 0] = 1
    W = bits_of(np.zeros((d_out, d_in)))
    ads = []
    for i in range(S):
        Af = np.zeros((2, d_in), np.float32); Af[0, 0] = 1
        Bf = np.zeros((d_out, 2), np.float32); Bf[:, 0] = i + 1
        ads.append(oracle.Adapter(oracle.LORA, 2, 1.0, bits_of(Af), bits_of(Bf)))
    _, Y = oracle.forward(off, ads, bits_of(Xf), W)
    seg = oracle.row_segment_map(off)
    expect = np.repeat(np.arange(S), lens)
    np.testing.assert_array_equal(seg, expect)
    np.testing.assert_array_equal(Y, (expect[:, None] + 1.0) * np.ones((1, d_out)))


def test_offsets_validation():
    for bad in ([1, 2], [0, 3, 2], [0, -1]):
        with pytest.raises(ValueError):
            oracle.row_segment_map(np.array(bad, dtype=np.int32))
    assert oracle.row_segment_map(np.array([0, 0, 0], dtype=np.int32)).size == 0


# ---------------------------------------------------------------------------
# P10: moments of the tiny configuration under the stated init laws
# ---------------------------------------------------------------------------
def test_cfg1_moments():
    wl = synth.cfg1_tiny()
    pr = wl.projections[0]
    X, W = synth.make_X(wl, pr), synth.make_W(wl, pr)
    ads = []
    for c in wl.clients:
        t = synth.make_adapter(wl, pr, c)
        ads.append(oracle.Adapter(t.kind, t.rank, t.scale, t.A, t.B))
    Y0, Y = oracle.forward(wl.offsets, ads, X, W)
    assert abs(np.var(Y0) - 1.0) < 0.05           # Var[x.w] = d_in * 1 * 1/d_in
    assert abs(np.var(Y) - 5.0) < 0.35            # + s^2 * r * (1/r) * d_in * (1/d_in), s = 2
    dY = synth.make_dY(wl, pr, wl.T)
    dXb = oracle.backward_input(wl.offsets, ads, dY, W, base_only=True)
    assert abs(np.var(dXb) - pr.d_out / pr.d_in) < 0.05


# ---------------------------------------------------------------------------
# IA3 gradient from the client's saved bf16 base output (Sec. 3.2: fine-tuning clients
# save the layer output for backward; Sec. 4: 16-bit).
# ---------------------------------------------------------------------------
def test_ia3_grad_from_saved_output():
    rng = np.random.default_rng(33)
    d_in, d_out = 3, 4
    off = np.array([0, 2, 7], dtype=np.int32)
    pick = lambda shape: bits_of(rng.choice([-1.0, -0.5, 0.0, 0.5, 1.0], size=shape))
    X, W, b, dY = pick((7, d_in)), pick((d_out, d_in)), pick((d_out,)), grid_bits(rng, (7, d_out))
    ads = [oracle.Adapter(oracle.LORA, 1, 1.0, pick((1, d_in)), pick((d_out, 1))),
           oracle.Adapter(oracle.IA3, 0, 0.0, grid_bits(rng, (d_out,)))]
    Y0, _ = oracle.forward(off, ads, X, W, b)
    # here every Y0 is a small multiple of 1/4, hence exact in bf16: both routes must agree exactly
    saved = bits_of(Y0)
    np.testing.assert_array_equal(oracle.ia3_grad(off, ads, X, dY, W, b, 1, Y0_saved=saved),
                                  oracle.ia3_grad(off, ads, X, dY, W, b, 1))
    # and with an arbitrary saved tensor the sum is over exactly that tensor (exact rationals)
    other = grid_bits(rng, (7, d_out))
    got = oracle.ia3_grad(off, ads, X, dY, W, b, 1, cols=[3, 1], Y0_saved=other)
    for q, j in enumerate([3, 1]):
        ref = sum(Fraction(float(f64(dY)[t, j])) * Fraction(float(f64(other)[t, j])) for t in range(2, 7))
        assert got[q] == float(ref)


def test_ia3_in_grad_from_saved_input_gradient():
    """IA3 input scaling: dl[k] = sum_t X[t][k] G[t][k] with G = dY W.  With the G the executor returned
    (a bf16 tensor) exactly representable, the saved route equals the recomputing one; with an arbitrary
    saved tensor the sum runs over exactly that tensor."""
    rng = np.random.default_rng(34)
    d_in, d_out = 4, 3
    off = np.array([0, 3, 7], dtype=np.int32)
    pick = lambda shape: bits_of(rng.choice([-1.0, -0.5, 0.0, 0.5, 1.0], size=shape))
    X, W, dY = grid_bits(rng, (7, d_in)), pick((d_out, d_in)), pick((7, d_out))
    ads = [oracle.Adapter(), oracle.Adapter(oracle.IA3_IN, 0, 0.0, grid_bits(rng, (d_in,)))]
    G = oracle.backward_input(off, ads, dY, W, base_only=True)        # dY W: small multiples of 1/4
    saved = bits_of(G)
    np.testing.assert_array_equal(oracle.ia3_grad(off, ads, X, dY, W, None, 1, G_saved=saved),
                                  oracle.ia3_grad(off, ads, X, dY, W, None, 1))
    other = grid_bits(rng, (7, d_in))
    got = oracle.ia3_grad(off, ads, X, dY, W, None, 1, cols=[2, 0], G_saved=other)
    for q, k in enumerate([2, 0]):
        ref = sum(Fraction(float(f64(X)[t, k])) * Fraction(float(f64(other)[t, k])) for t in range(3, 7))
        assert got[q] == float(ref)
