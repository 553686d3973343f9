"""Pins for the oracle's variants: fixed-count (top-k) activation, the signed threshold, an output bias, and the
multi-phase activation with its residual biases (R-Sparse, Sec. 3.2).  CPU only; none of these compares the oracle
with itself: numpy's sort and matvec, literal loops, a hand-worked example and the identities the paper states."""
import os

import numpy as np
import pytest

import oracle
from paper_2504_19449_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- fixed-count activation

def _topk_by_numpy(x, k):
    """Stable selection with numpy: sort by (-|x|, index); NaN excluded."""
    x = np.asarray(x, dtype=np.float64)
    idx = np.arange(len(x))
    ok = ~np.isnan(x)
    order = np.lexsort((idx[ok], -np.abs(x[ok])))           # last key is the primary one
    m = np.zeros(len(x), dtype=np.uint8)
    m[idx[ok][order[:k]]] = 1
    return m


@pytest.mark.parametrize("dtype", [synth.F16, synth.BF16])
def test_topk_mask_against_numpy_sort(dtype):
    g = _rng(11)
    for d in (8, 64, 1000):
        x16 = synth.encode16(g.laplace(size=d) * np.exp(g.standard_normal(d)), dtype)      # 16-bit values: ties occur
        x16[::7] = x16[3]                                                                  # and are planted
        for k in (0, 1, 2, d // 3, d // 2, d - 1, d, d + 5):
            got = oracle.topk_mask(x16, dtype, k)
            want = _topk_by_numpy(synth.decode16(x16, dtype), k)
            assert np.array_equal(got, want), (d, k)
            assert got.sum() == min(k, d)


def test_topk_ties_go_to_the_lower_channel_and_nan_is_never_kept():
    x = np.array([1.0, -3.0, 3.0, np.nan, 3.0, -1.0, 0.0, -0.0])
    assert oracle.topk_mask(x, oracle.F64, 1).tolist() == [0, 1, 0, 0, 0, 0, 0, 0]
    assert oracle.topk_mask(x, oracle.F64, 2).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]
    assert oracle.topk_mask(x, oracle.F64, 3).tolist() == [0, 1, 1, 0, 1, 0, 0, 0]
    assert oracle.topk_mask(x, oracle.F64, 4).tolist() == [1, 1, 1, 0, 1, 0, 0, 0]
    assert oracle.topk_mask(x, oracle.F64, 6).tolist() == [1, 1, 1, 0, 1, 1, 1, 0]
    assert oracle.topk_mask(x, oracle.F64, 8).tolist() == [1, 1, 1, 0, 1, 1, 1, 1]           # 7 non-NaN channels
    inf = np.array([1.0, np.inf, -np.inf, 2.0])
    assert oracle.topk_mask(inf, oracle.F64, 2).tolist() == [0, 1, 1, 0]


def test_topk_equals_the_threshold_mask_when_the_boundary_has_no_tie():
    g = _rng(5)
    x = g.standard_normal(257)                                  # fp64 draws: no ties
    a = np.sort(np.abs(x))[::-1]
    for k in (1, 17, 128, 257):
        tau = np.float32(a[k - 1])                              # may round; pick tau strictly between neighbours instead
        lo = a[k] if k < len(a) else 0.0
        tau = np.float32((a[k - 1] + lo) / 2)
        assert lo < float(tau) < a[k - 1]
        assert np.array_equal(oracle.topk_mask(x, oracle.F64, k), oracle.mask(x, oracle.F64, tau))


def test_layer_with_topk_is_the_masked_layer_and_matches_numpy():
    L = synth.make_layer(48, 40, 8, synth.BF16, config=9, linear=1)
    X16 = synth.encode16(synth.DModelInput(48, config=9, linear=1).tokens(3), synth.BF16)
    k = 19
    out = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, synth.BF16, synth.BF16, 0.0, topk=k)
    W, U, SV, X = (synth.decode16(a, synth.BF16) for a in (L.W16, L.U16, L.SV16, X16))
    for b in range(3):
        m = _topk_by_numpy(X[b], k).astype(bool)
        assert np.array_equal(out["act"][b], np.nonzero(m)[0])
        want = W[:, m] @ X[b, m] + U @ (SV[:, ~m] @ X[b, ~m])
        assert np.allclose(out["Y"][b], want, rtol=1e-12, atol=1e-13)
    assert np.array_equal(out["union"], np.nonzero(np.any([_topk_by_numpy(X[b], k) for b in range(3)], axis=0))[0])


# ---------------------------------------------------------------- signed threshold, bias

def test_signed_threshold_by_a_literal_loop():
    x = np.array([-2.0, -0.5, 0.0, -0.0, 0.5, 1.0, np.nan, np.inf, -np.inf])
    for tau in (-1.0, 0.0, 0.5, 1.0):
        want = [1 if (v >= tau) else 0 for v in x]              # NaN compares false
        assert oracle.mask(x, oracle.F64, tau, cmp_mode=2).tolist() == want


def test_bias_is_added_once_to_every_token():
    L = synth.make_layer(32, 24, 8, synth.F16, config=9, linear=2)
    X16 = synth.encode16(synth.DModelInput(32, config=9, linear=2).tokens(2), synth.F16)
    bias = _rng(3).standard_normal(24)
    a = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, synth.F16, synth.F16, 0.7)
    b = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, synth.F16, synth.F16, 0.7, bias=bias)
    assert np.allclose(b["Y"] - a["Y"], bias[None, :], rtol=0, atol=1e-13)
    assert all(np.array_equal(p, q) for p, q in zip(a["act"], b["act"]))


def test_masked_core_with_arbitrary_masks_against_numpy():
    g = _rng(8)
    d_in, d_out, r = 20, 12, 5
    W, U, SV = g.standard_normal((d_out, d_in)), g.standard_normal((d_out, r)), g.standard_normal((r, d_in))
    X = g.standard_normal((4, d_in))
    M = (g.random((4, d_in)) < 0.4).astype(np.uint8)
    M[2] = 0
    M[3] = 1
    Y = oracle.rsparse_linear_masked(W, U, SV, X, oracle.F64, oracle.F64, M)
    want = (X * M) @ W.T + ((X * (1 - M)) @ SV.T) @ U.T
    assert np.allclose(Y, want, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- Sec. 3.2: multi-phase activation

def _golden():
    out = {}
    for line in open(os.path.join(GOLDEN, "hand_worked_multiphase.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = np.array([float(v) for v in vals])
    return out


def test_multiphase_hand_worked_example():
    gd = _golden()
    T, W, h = gd["T"], gd["W"].reshape(2, 5), gd["h"]
    assert np.array_equal(oracle.multiphase(h, T), gd["sigma"])
    Yr, B = oracle.multiphase_residual(W, oracle.F64, h, oracle.F64, T)
    assert np.array_equal(B[0], gd["B0"]) and np.array_equal(B[1], gd["B1"])
    assert np.array_equal(Yr, gd["Yr"])
    # the sparse part is the layer with the signed threshold T_0 and no low-rank part
    Ys = oracle.rsparse_linear(W, None, None, h, oracle.F64, oracle.F64, T[0], cmp_mode=2)["Y"][0]
    assert np.array_equal(Ys, gd["Ys"])
    assert np.array_equal(Ys + Yr, gd["Y"])


def test_multiphase_with_one_phase_at_zero_is_relu():
    x = _rng(2).standard_normal(500)
    assert np.array_equal(oracle.multiphase(x, [0.0]), np.maximum(x, 0.0))
    Yr, _ = oracle.multiphase_residual(np.ones((3, 500)), oracle.F64, x, oracle.F64, [0.0])
    assert np.array_equal(Yr, np.zeros(3))


def test_sparse_part_plus_residual_is_the_layer_on_the_multiphase_input():
    """Sec. 3.2's decomposition: Y_s + Y_r = sigma_T(H) W^T (numpy's matvec on numpy's own piecewise function)."""
    g = _rng(21)
    d_in, d_out = 300, 40
    W = g.standard_normal((d_out, d_in))
    for l in (1, 2, 3, 5):
        h = g.standard_normal(d_in) * 1.5
        T = np.sort(g.uniform(-1.0, 1.0, size=l))[::-1].copy()
        T[-1] = min(T[-1], h.min()) if l > 1 else T[-1]          # the paper's choice: T_{l-1} = the input's minimum
        T = np.array(sorted(set(T), reverse=True))
        sig = np.where(h >= T[0], h, 0.0)
        for i in range(len(T) - 1):
            sig = np.where((h < T[i]) & (h >= T[i + 1]), 0.5 * (T[i] + T[i + 1]), sig)
        assert np.allclose(oracle.multiphase(h, T), sig, rtol=0, atol=0)
        Yr, B = oracle.multiphase_residual(W, oracle.F64, h, oracle.F64, T)
        Ys = oracle.rsparse_linear(W, None, None, h, oracle.F64, oracle.F64, T[0], cmp_mode=2)["Y"][0]
        assert np.allclose(Ys + Yr, W @ sig, rtol=1e-11, atol=1e-11)
        for i in range(len(T) - 1):                               # each bias is a plain column sum
            sel = (h < T[i]) & (h >= T[i + 1])
            assert np.allclose(B[i], W[:, sel].sum(axis=1), rtol=1e-12, atol=1e-12)


def test_static_bias_is_the_mean_residual_and_linear_in_w():
    g = _rng(33)
    d_in, d_out, N = 64, 16, 9
    W16 = synth.encode16(g.standard_normal((d_out, d_in)) * 0.1, synth.BF16)
    H16 = synth.encode16(g.standard_normal((N, d_in)), synth.BF16)
    T = np.array([0.5, -0.25, -4.0])
    b = oracle.static_bias(W16, synth.BF16, H16, synth.BF16, T)
    W, H = synth.decode16(W16, synth.BF16), synth.decode16(H16, synth.BF16)
    # one token: its own residual
    one = oracle.static_bias(W16, synth.BF16, H16[:1], synth.BF16, T)
    assert np.array_equal(one, oracle.multiphase_residual(W16, synth.BF16, H16[0], synth.BF16, T)[0])
    # N tokens: W times the mean of the residual part of sigma_T(H)
    res = np.where(H >= T[0], 0.0, np.where(H >= T[1], 0.5 * (T[0] + T[1]), 0.5 * (T[1] + T[2])))
    assert np.allclose(b, W @ res.mean(axis=0), rtol=1e-12, atol=1e-13)
