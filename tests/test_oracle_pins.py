"""Pins for the CPU oracle: every check compares it with something the paper or the
mathematics fixes, computed *without* the oracle's own formula path -- numpy's matvec,
closed-form singular factors from the generator, literal Python loops over the
(singular component, channel) double sum of Sec. 3.3, order-statistic definitions.

Rectangular layers are used throughout so that a transposed operand fails.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from paper_2504_19449_amd import synth

INF = float("inf")


# --------------------------------------------------------------------------- storage formats

def test_fp16_decode_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode16(bits, oracle.F16)
    want = bits.view(np.float16).astype(np.float64)       # numpy's own half decoder
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))
    # fp16 subnormals are kept, not flushed (Sec. 3.4 stores W as is)
    assert got[1] == 2.0 ** -24 and got[0x03FF] == 1023 * 2.0 ** -24


def test_bf16_decode_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode16(bits, oracle.BF16)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])


# --------------------------------------------------------------------------- hand-worked example

def _read_golden(path):
    """Parse tests/golden/*.txt: 'case:' starts a case, 'key: numbers' lines fill it (rows split by ';')."""
    cases, cur = [], None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, val = (p.strip() for p in line.split(":", 1))
        if key == "case":
            cur = {"name": val, "expect": []}
            cases.append(cur)
            continue
        rows = [[float(v) for v in row.split()] for row in val.split(";")]
        if key.startswith("expect"):
            _, cmp_s, union_s, what = key.split()
            cur["expect"].append((int(cmp_s.split("=")[1]), int(union_s.split("=")[1]), what, rows))
        else:
            cur[key] = rows
    return cases


def test_hand_worked_golden():
    """Cases worked by hand from the definition of Sec. 3.4 (ties, strict compare, two tokens with
    different masks, rank 2, union mode); the fixture states how each number was obtained."""
    path = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_sec3_4.txt")
    cases = _read_golden(path)
    assert [c["name"] for c in cases] == ["tie_2x3", "batch2_rank2_3x4"]
    for c in cases:
        W, U, SV, X = (np.array(c[k], dtype=np.float64) for k in ("W", "U", "SV", "X"))
        tau = c["tau"][0][0]
        assert c["expect"], c["name"]
        for cmp_mode, union, what, rows in c["expect"]:
            out = oracle.rsparse_linear(W, U, SV, X, oracle.F64, oracle.F64, tau, cmp_mode=cmp_mode,
                                        batch_mask_mode=union)
            if what == "kept":
                if union:
                    assert out["union"].tolist() == [int(v) for v in rows[0]], (c["name"], cmp_mode)
                else:
                    assert [a.tolist() for a in out["act"]] == [[int(v) for v in r] for r in rows], \
                        (c["name"], cmp_mode)
            else:
                assert out["Y"].tolist() == rows, (c["name"], cmp_mode, union)


# --------------------------------------------------------------------------- mask / index sets

def test_mask_literal_loop_all_reachable_thresholds():
    rng = np.random.default_rng(5)
    x = rng.permutation(np.arange(1, 9)).astype(np.float64) * rng.choice([-1, 1], 8)
    mags = sorted(abs(x))
    taus = [-INF, 0.0] + mags + [(a + b) / 2 for a, b in zip(mags, mags[1:])] + [9.0, INF]
    for tau in taus:
        for mode in (0, 1):
            want = [c for c in range(8) if (abs(x[c]) >= tau if mode == 0 else abs(x[c]) > tau)]
            got = oracle.rsparse_linear(np.eye(8), None, None, x, oracle.F64, oracle.F64, tau,
                                        cmp_mode=mode)
            assert got["act"][0].tolist() == want
            assert oracle.mask(x, oracle.F64, tau, mode).tolist() == [int(c in want) for c in range(8)]


def test_mask_special_values_f16():
    # NaN is never kept, +-Inf always (for finite tau), -0 is 0; all-ties token under both modes
    x = np.array([np.nan, np.inf, -np.inf, -0.0, 0.0, 1.0, -1.0, 6e-8], dtype=np.float16)
    bits = x.view(np.uint16)
    assert oracle.mask(bits, oracle.F16, 1.0, 0).tolist() == [0, 1, 1, 0, 0, 1, 1, 0]
    assert oracle.mask(bits, oracle.F16, 1.0, 1).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]
    assert oracle.mask(bits, oracle.F16, 0.0, 0).tolist() == [0, 1, 1, 1, 1, 1, 1, 1]
    assert oracle.mask(bits, oracle.F16, 0.0, 1).tolist() == [0, 1, 1, 0, 0, 1, 1, 1]
    assert oracle.mask(bits, oracle.F16, -INF, 0).tolist() == [0, 1, 1, 1, 1, 1, 1, 1]
    assert oracle.mask(bits, oracle.F16, INF, 0).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]
    assert oracle.mask(bits, oracle.F16, INF, 1).tolist() == [0] * 8
    ties = synth.encode16(np.array([0.75, -0.75] * 8), synth.F16)
    assert oracle.mask(ties, oracle.F16, 0.75, 0).sum() == 16
    assert oracle.mask(ties, oracle.F16, 0.75, 1).sum() == 0


# --------------------------------------------------------------------------- special cases that reduce to a matvec

def _x_for(layer, n=3, seed=0):
    src = synth.DModelInput(layer.d_in, config=91, linear=seed)
    return synth.encode16(src.tokens(n), layer.dtype)


def _dec(layer):
    return (synth.decode16(layer.W16, layer.dtype), synth.decode16(layer.U16, layer.dtype),
            synth.decode16(layer.SV16, layer.dtype))


@pytest.mark.parametrize("name", ["wide_f16", "tall_bf16", "square_f16"])
def test_all_active_equals_dense_for_every_rank(small_layers, name):
    L = small_layers[name]
    X16 = _x_for(L)
    Wd, _, _ = _dec(L)
    want = synth.decode16(X16, L.dtype) @ Wd.T                      # numpy fp64 matvec
    for r in (0, 1, L.rank):
        got = oracle.rsparse_linear(L.W16, L.U16[:, :r], L.SV16[:r], X16, L.dtype, L.dtype, -INF)
        assert np.allclose(got["Y"], want, rtol=1e-12, atol=1e-13)
        assert all(a.tolist() == list(range(L.d_in)) for a in got["act"])
    assert np.allclose(oracle.dense_linear(L.W16, X16, L.dtype, L.dtype), want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("name", ["wide_f16", "tall_bf16"])
def test_rank_zero_is_sparse_only(small_layers, name):
    L = small_layers[name]
    X16 = _x_for(L, seed=1)
    Wd, _, _ = _dec(L)
    Xd = synth.decode16(X16, L.dtype)
    tau = float(np.float32(np.median(np.abs(Xd))))
    got = oracle.rsparse_linear(L.W16, None, None, X16, L.dtype, L.dtype, tau)
    keep = np.abs(Xd) >= tau
    assert np.allclose(got["Y"], (Xd * keep) @ Wd.T, rtol=1e-12, atol=1e-13)
    for b in range(Xd.shape[0]):
        assert got["act"][b].tolist() == np.flatnonzero(keep[b]).tolist()
    # linearity: the kept part plus the dropped part (run with everything active) is the dense product
    rest = oracle.rsparse_linear(Wd, None, None, Xd * ~keep, oracle.F64, oracle.F64, -INF)
    assert np.allclose(got["Y"] + rest["Y"], Xd @ Wd.T, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("name", ["wide_f16", "tall_bf16"])
def test_none_active_is_low_rank_only_closed_form(small_layers, name):
    """tau = +inf routes every channel through the rank-r path: Y = U_r diag(s_r) V_r^T x with the
    generator's closed-form factors (unrounded float64 operands on both sides)."""
    L = small_layers[name]
    Xd = synth.DModelInput(L.d_in, config=91, linear=2).tokens(3)
    r = L.rank
    W = (L.U * L.sigma) @ L.V.T
    U_r = L.U[:, :r]
    SV_r = (L.V[:, :r] * L.sigma[:r]).T
    got = oracle.rsparse_linear(W, U_r, SV_r, Xd, oracle.F64, oracle.F64, INF)
    want = np.stack([sum(L.sigma[i] * (L.V[:, i] @ x) * L.U[:, i] for i in range(r)) for x in Xd])
    assert np.allclose(got["Y"], want, rtol=1e-11, atol=1e-13)
    assert all(len(a) == 0 for a in got["act"])
    # and with the stored 16-bit factors: plain numpy on the decoded bits
    Wd, Ud, SVd = _dec(L)
    X16 = synth.encode16(Xd, L.dtype)
    got16 = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, L.dtype, L.dtype, INF)
    assert np.allclose(got16["Y"], (synth.decode16(X16, L.dtype) @ SVd.T) @ Ud.T, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("name", ["wide_f16", "tall_bf16"])
def test_full_rank_equals_dense_for_any_mask(small_layers, name):
    L = small_layers[name]
    p = min(L.d_in, L.d_out)
    W = (L.U * L.sigma) @ L.V.T
    SV = (L.V * L.sigma).T
    Xd = synth.DModelInput(L.d_in, config=91, linear=3).tokens(4)
    for tau in (0.3, 1.0, 5.0, INF):
        got = oracle.rsparse_linear(W, L.U[:, :p], SV[:p], Xd, oracle.F64, oracle.F64, tau)
        assert np.allclose(got["Y"], Xd @ W.T, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- the double sum of Sec. 3.3

def _double_sum(U, sigma, V, x, kept_channels, r):
    """Y = sum_i sum_j sigma_i x_j V[j,i] U[:,i] over the kept (i, j) pairs: every i for a kept
    channel j, and i < r for the others -- the score matrix with its low-sigma / low-|x|
    corner removed (Sec. 3.3 - 3.4).  Literal loops."""
    n_out, p = U.shape
    y = [0.0] * n_out
    for j in range(len(x)):
        top = p if j in kept_channels else r
        for i in range(top):
            s_ij = sigma[i] * x[j] * V[j, i]
            for o in range(n_out):
                y[o] += s_ij * U[o, i]
    return np.array(y)


def test_double_sum_brute_force_all_masks_8x8():
    L = synth.make_layer(8, 8, 0, synth.F16, config=92, linear=0)
    W = (L.U * L.sigma) @ L.V.T
    rng = np.random.default_rng(11)
    worst = 0.0
    for mask_bits in range(256):
        kept = {c for c in range(8) if (mask_bits >> c) & 1}
        big = rng.uniform(1.5, 3.0, 8) * rng.choice([-1, 1], 8)
        small = rng.uniform(0.05, 0.9, 8) * rng.choice([-1, 1], 8)
        x = np.array([big[c] if c in kept else small[c] for c in range(8)])
        for r in range(9):
            got = oracle.rsparse_linear(W, L.U[:, :r], (L.V[:, :r] * L.sigma[:r]).T, x,
                                        oracle.F64, oracle.F64, 1.0)
            assert set(got["act"][0].tolist()) == kept
            want = _double_sum(L.U, L.sigma, L.V, x, kept, r)
            worst = max(worst, np.max(np.abs(got["Y"][0] - want)))
    assert worst < 1e-12


def test_double_sum_rectangular():
    for d_in, d_out in ((10, 6), (5, 9)):
        L = synth.make_layer(d_in, d_out, 0, synth.F16, config=92, linear=d_in)
        W = (L.U * L.sigma) @ L.V.T
        x = synth.DModelInput(d_in, config=92, linear=1).tokens(1)[0]
        tau = float(np.float32(np.median(np.abs(x))))
        kept = {c for c in range(d_in) if abs(x[c]) >= tau}
        for r in range(min(d_in, d_out) + 1):
            got = oracle.rsparse_linear(W, L.U[:, :r], (L.V[:, :r] * L.sigma[:r]).T, x,
                                        oracle.F64, oracle.F64, tau)
            assert np.allclose(got["Y"][0], _double_sum(L.U, L.sigma, L.V, x, kept, r),
                               rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- error bound

def test_eckart_young_bound(small_layers):
    """||Y_rsparse - W x||_2 <= sigma_{r+1} ||x (.) not-m||_2: the dropped block is the tail of the
    SVD applied to the dropped channels."""
    L = small_layers["wide_f16"]
    W = (L.U * L.sigma) @ L.V.T
    Xd = synth.DModelInput(L.d_in, config=91, linear=4).tokens(5)
    for r in (0, 3, 12, 30):
        for tau in (0.2, 1.0, 3.0, INF):
            got = oracle.rsparse_linear(W, L.U[:, :r], (L.V[:, :r] * L.sigma[:r]).T, Xd,
                                        oracle.F64, oracle.F64, tau)
            err = np.linalg.norm(got["Y"] - Xd @ W.T, axis=1)
            dropped = np.linalg.norm(Xd * (np.abs(Xd) < tau), axis=1)
            assert np.all(err <= L.sigma[r] * dropped * (1 + 1e-9) + 1e-12)
            if r > 0 and tau > 0.2:
                assert np.any(err > 1e-6)      # the approximation really is one


# --------------------------------------------------------------------------- batch semantics

def test_batch_is_independent_tokens_and_union(small_layers):
    L = small_layers["tall_bf16"]
    X16 = _x_for(L, n=5, seed=5)
    tau = float(np.float32(0.8))
    both = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, L.dtype, L.dtype, tau)
    for b in range(5):
        one = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16[b], L.dtype, L.dtype, tau)
        assert np.array_equal(one["Y"][0], both["Y"][b])
        assert one["act"][0].tolist() == both["act"][b].tolist()
    uni = sorted(set().union(*[set(a.tolist()) for a in both["act"]]))
    assert both["union"].tolist() == uni
    # union-mask mode: every token keeps the union's channels
    um = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, L.dtype, L.dtype, tau, batch_mask_mode=1)
    Wd, Ud, SVd = _dec(L)
    Xd = synth.decode16(X16, L.dtype)
    keep = np.zeros(L.d_in, bool)
    keep[uni] = True
    want = (Xd * keep) @ Wd.T + ((Xd * ~keep) @ SVd.T) @ Ud.T
    assert np.allclose(um["Y"], want, rtol=1e-11, atol=1e-14)
    assert all(a.tolist() == uni for a in um["act"])


def test_threads_do_not_change_the_result(small_layers):
    L = small_layers["wide_f16"]
    X16 = _x_for(L, n=2, seed=6)
    a = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, L.dtype, L.dtype, 0.7, nthreads=1)
    b = oracle.rsparse_linear(L.W16, L.U16, L.SV16, X16, L.dtype, L.dtype, 0.7, nthreads=4)
    assert np.array_equal(a["Y"], b["Y"])


# --------------------------------------------------------------------------- threshold estimation

@pytest.mark.parametrize("s", [0.0, 0.25, 0.4, 0.5, 0.7, 0.999, 1.0])
def test_quantile_tau_is_the_order_statistic(s):
    src = synth.DModelInput(256, config=93, linear=0)
    X16 = synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), synth.F16)
    tau = oracle.quantile_tau(X16, oracle.F16, s)
    a = np.abs(synth.decode16(X16, synth.F16)).ravel()
    n = a.size
    target = min(int(math.floor(s * n)), n - 1)
    assert tau == np.sort(a)[target]
    assert tau == np.partition(a, target)[target]
    assert np.sum(a < tau) <= target <= np.sum(a <= tau) - 1 + (1 if s == 1.0 else 0) or s == 1.0
    # tau is a 16-bit value, hence exact in fp32
    assert float(np.float32(tau)) == tau
    if 0 < s < 1:
        frac = np.mean(a < tau)
        assert abs(frac - s) < 2e-3


# --------------------------------------------------------------------------- gated MLP input (Sec. 3.1)

def test_silu32_recipe_against_fp64():
    """The fp32 recipe that defines the activation stays within a few ulp of g / (1 + exp(-g))."""
    g = np.concatenate([np.linspace(-87.0, 87.0, 400001), np.random.default_rng(3).standard_normal(200000) * 3.0,
                        np.array([0.0, -0.0, 1e-30, -1e-30, 1e-3, 20.0, 60.0, 88.0, 1e30])]).astype(np.float32)
    got = oracle.silu32(g).astype(np.float64)
    g64 = g.astype(np.float64)
    want = g64 / (1.0 + np.exp(-g64))
    ulp = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
    assert np.max(np.abs(got - want) / ulp) <= 3.0          # measured: 2.4
    # special values
    sp = oracle.silu32(np.array([np.nan, np.inf, -np.inf, -88.0, -1e30, 0.0], dtype=np.float32))
    assert np.isnan(sp[0]) and sp[1] == np.inf
    assert all(v == 0.0 and np.signbit(v) for v in sp[2:5])
    assert sp[5] == 0.0
    # shape of the function: minimum about -0.2785 near g = -1.2785, identity for large g
    dense = oracle.silu32(np.linspace(-10, 10, 20001).astype(np.float32))
    assert abs(dense.min() + 0.27846) < 1e-4 and abs(np.linspace(-10, 10, 20001)[dense.argmin()] + 1.2785) < 2e-3
    assert oracle.silu32(np.array([50.0], dtype=np.float32))[0] == 50.0


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_gated_input_is_one_rounding_of_the_fp32_product(dt):
    """h = round16(silu32(g) * u): the multiply and the single rounding, against numpy's own fp32
    product and 16-bit conversions (synth.encode16), including fp16 subnormals, overflow and NaN."""
    rng = np.random.default_rng(11)
    g = rng.standard_normal(100000) * 2.0
    u = rng.standard_normal(100000) * np.exp(rng.uniform(-12, 8, 100000))      # wide range: subnormals to overflow
    g[:4] = [np.nan, 1.0, 3.0, -2.0]
    u[:4] = [1.0, np.nan, np.inf, 60000.0]
    G16, U16 = synth.encode16(g, dt), synth.encode16(u, dt)
    got = oracle.gated_input(G16, U16, dt)
    gf = synth.decode16(G16, dt).astype(np.float32)
    uf = synth.decode16(U16, dt).astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        want = synth.encode16(oracle.silu32(gf) * uf, dt)
    nan = np.isnan(synth.decode16(want, dt))
    assert np.array_equal(np.isnan(synth.decode16(got, dt)), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert nan[:2].all() and np.isinf(synth.decode16(got[2:3], dt))[0]


def _boundary_words():
    """fp32 bit patterns that exercise a 16-bit rounding: every high half with the low half at 0, just below
    half, exactly half and just above half (ties, carries into the exponent, overflow to infinity, NaN and
    infinity included), plus a million random words."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x7FFF, 0x8000, 0x8001, 0x0001, 0xFFFF, 0x1000, 0x0FFF, 0x1001, 0x2FFF, 0x3000], dtype=np.uint32)
    words = (hi[:, None] | lows[None, :]).reshape(-1)
    rnd = np.random.default_rng(5).integers(0, 2 ** 32, size=1_000_000, dtype=np.uint64).astype(np.uint32)
    return np.concatenate([words, rnd])


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_fp32_to_16bit_rounding_against_torch(dt):
    """The oracle's fp32 -> bf16 / fp16 roundings against torch's CPU conversions (an implementation of its
    own: neither the add-0x7FFF formula of the generators nor the device's), bit for bit on every non-NaN
    input; NaN must stay NaN."""
    import torch
    f = _boundary_words().view(np.float32)
    got = oracle.round16(f, dt)
    tdt = torch.float16 if dt == synth.F16 else torch.bfloat16
    want = torch.from_numpy(f.copy()).to(tdt).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan])
    dec = synth.decode16(got[nan], dt)
    assert np.isnan(dec).all()
    # the overflow edge in words: the largest fp32 values below the rounding point stay finite, the rest become inf
    if dt == synth.BF16:
        assert oracle.round16(np.array([0x7F7F7FFF], dtype=np.uint32).view(np.float32), dt)[0] == 0x7F7F
        assert oracle.round16(np.array([0x7F7F8000], dtype=np.uint32).view(np.float32), dt)[0] == 0x7F80
    else:
        assert oracle.round16(np.array([65519.996], dtype=np.float32), dt)[0] == 0x7BFF
        assert oracle.round16(np.array([65520.0], dtype=np.float32), dt)[0] == 0x7C00


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_fp64_to_16bit_rounding_by_definition(dt):
    """round16_from_double (used by the plain-definition gated input) against (a) torch on doubles that are
    exact fp32 values, (b) exact rational arithmetic on random doubles: the result is a nearest representable
    neighbour, ties to the even one, (c) doubles a hair above / below a tie, which a double rounding through
    fp32 would get wrong."""
    import torch
    from fractions import Fraction
    f = _boundary_words()[:65536 * 11:7].view(np.float32)
    tdt = torch.float16 if dt == synth.F16 else torch.bfloat16
    want = torch.from_numpy(f.copy()).to(tdt).view(torch.int16).numpy().view(np.uint16)
    got = oracle.round16_from_double(f.astype(np.float64), dt)
    ok = ~np.isnan(f)
    assert np.array_equal(got[ok], want[ok])
    # (b) exact check on random doubles over the whole finite range of the format
    rng = np.random.default_rng(8)
    top = 17.0 if dt == synth.F16 else 128.5
    low = -26.0 if dt == synth.F16 else -136.0
    v = np.ldexp(rng.uniform(1.0, 2.0, 3000), rng.integers(int(low), int(top), 3000)) * rng.choice([-1.0, 1.0], 3000)
    bits = oracle.round16_from_double(v, dt)
    dec = synth.decode16(bits, dt)
    allv = np.sort(synth.decode16(np.arange(65536, dtype=np.uint16), dt))
    allv = allv[np.isfinite(allv)]
    for x, b, d in zip(v, bits, dec):
        i = np.searchsorted(allv, x)
        cands = [allv[j] for j in (i - 1, i) if 0 <= j < len(allv)]
        if np.isinf(d):
            # overflow: x is at least half a spacing past the largest finite value
            big = Fraction(float(allv[-1]))
            sp = big - Fraction(float(allv[-2]))
            assert abs(Fraction(float(x))) >= big + sp / 2
            continue
        err = abs(Fraction(float(d)) - Fraction(float(x)))
        best = min(abs(Fraction(float(c)) - Fraction(float(x))) for c in cands)
        assert err == best, (x, d, cands)
        if len(cands) == 2 and abs(Fraction(float(cands[0])) - Fraction(float(x))) == abs(Fraction(float(cands[1])) - Fraction(float(x))):
            assert (int(b) & 1) == 0
    # (c) ties and near-ties
    one = 1.0
    sp = 2.0 ** -10 if dt == synth.F16 else 2.0 ** -7
    up_bits = oracle.round16_from_double(np.array([one + sp]), dt)[0]
    one_bits = oracle.round16_from_double(np.array([one]), dt)[0]
    two_bits = oracle.round16_from_double(np.array([one + 2 * sp]), dt)[0]
    mid = one + sp / 2
    assert oracle.round16_from_double(np.array([mid]), dt)[0] == one_bits                  # tie -> even (1.0)
    assert oracle.round16_from_double(np.array([np.nextafter(mid, 2.0)]), dt)[0] == up_bits
    assert oracle.round16_from_double(np.array([one + 1.5 * sp]), dt)[0] == two_bits       # tie -> even (1 + 2 sp)
    assert oracle.round16_from_double(np.array([np.nextafter(one + 1.5 * sp, 0.0)]), dt)[0] == up_bits
    # a value that rounds to the tie in fp32 first and then the wrong way: mid + 2^-30 must go up
    assert oracle.round16_from_double(np.array([mid + 2.0 ** -30]), dt)[0] == up_bits
    # signed zero, infinities, subnormal spacing
    z = oracle.round16_from_double(np.array([0.0, -0.0, np.inf, -np.inf]), dt)
    assert list(z) == ([0x0000, 0x8000, 0x7C00, 0xFC00] if dt == synth.F16 else [0x0000, 0x8000, 0x7F80, 0xFF80])
    tiny = 2.0 ** -24 if dt == synth.F16 else 2.0 ** -133
    assert list(oracle.round16_from_double(np.array([tiny, 0.5 * tiny, 0.5000001 * tiny, 1.5 * tiny, 2.5 * tiny]), dt)) == [1, 0, 1, 2, 2]


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_gated_input_plain_definition(dt):
    """The gated input by its definition (Sec. 3.1: the up projection times SiLU of the gate projection)
    against numpy's fp64 evaluation, a closed-form identity and special values; and the fp32 recipe that
    the index sets are built from differs from it only where the exact product sits next to a rounding flip
    point."""
    rng = np.random.default_rng(21)
    n = 200000
    g = rng.standard_normal(n) * 3.0
    u = rng.standard_normal(n) * np.exp(rng.uniform(-6, 4, n))
    G16, U16 = synth.encode16(g, dt), synth.encode16(u, dt)
    bits, margin = oracle.gated_input_plain(G16, U16, dt)
    gd, ud = synth.decode16(G16, dt), synth.decode16(U16, dt)
    # numpy: g * sigmoid(g) with the logistic written the other way round (1 / (1 + e^-g) = e^g / (1 + e^g))
    with np.errstate(over="ignore"):
        ref = ud * gd * np.where(gd >= 0, 1.0 / (1.0 + np.exp(-gd)), np.exp(gd) / (1.0 + np.exp(gd)))
    want = oracle.round16_from_double(ref, dt)
    differ = bits != want
    assert differ.mean() < 1e-6 and (margin[differ] < 1e-9).all()      # only exact-tie hair-splitting between the two fp64 forms
    # identity silu(g) - silu(-g) = g  (from sigmoid(g) + sigmoid(-g) = 1), checked on the unrounded path via u = 1
    ones = synth.encode16(np.ones(1000), dt)
    gp = synth.encode16(np.linspace(0.01, 8.0, 1000), dt)
    gm = synth.encode16(-synth.decode16(gp, dt), dt)
    sp_ = synth.decode16(oracle.gated_input_plain(gp, ones, dt)[0], dt)
    sm_ = synth.decode16(oracle.gated_input_plain(gm, ones, dt)[0], dt)
    spacing = 2.0 ** (-10 if dt == synth.F16 else -7)
    assert np.all(np.abs((sp_ - sm_) - synth.decode16(gp, dt)) <= 1.01 * spacing * np.maximum(np.abs(sp_), 0.28))
    # special values: silu(0) = 0, silu(-inf) u = -0 * u, silu(+inf) = +inf, NaN propagates
    sv = oracle.gated_input_plain(synth.encode16(np.array([0.0, -np.inf, np.inf, np.nan, 2.0]), dt),
                                  synth.encode16(np.array([3.0, 2.0, 2.0, 1.0, np.nan]), dt), dt)[0]
    d = synth.decode16(sv, dt)
    assert d[0] == 0.0 and d[1] == 0.0 and np.signbit(d[1]) and d[2] == np.inf and np.isnan(d[3]) and np.isnan(d[4])
    # the fp32 recipe against the definition: equal bits wherever the exact product is not within the
    # recipe's error of a flip point.  The recipe is within 3 ulp (fp32) of silu and adds one fp32 rounding of
    # the product: <= 3.5 ulp <= 7 * 2^-24 relative, i.e. at most 7 * 2^-24 * 2^p of the 16-bit spacing
    # (p significand bits: the spacing is at least 2^-p of the value).
    recipe = oracle.gated_input(G16, U16, dt)
    p_bits = 11 if dt == synth.F16 else 8
    band = oracle.RECIPE_BAND[dt]
    finite = np.isfinite(synth.decode16(bits, dt))
    outside = finite & (margin > band)
    assert np.array_equal(recipe[outside], bits[outside])
    inside = finite & ~outside
    assert inside.mean() < 4 * band + 1e-3          # the band is a sliver of the number line
    # inside the band the two may differ by at most one step of the 16-bit grid
    a, b = synth.decode16(recipe[inside], dt), synth.decode16(bits[inside], dt)
    assert np.all(np.abs(a - b) <= 2.0 ** (1 - p_bits) * np.maximum(np.abs(a), np.abs(b)) + 1e-45)


# --------------------------------------------------------------------------- recipe search (Sec. 3.5)

def _quad(center):
    return lambda rho: float(sum((a - b) ** 2 for a, b in zip(rho, center)))


def test_recipe_search_invariants():
    """What the algorithm fixes regardless of its random draws: the best loss never gets worse from one
    generation to the next (lowest-loss selection over parents and offspring); with no generations the
    answer is the best of the initial population; with crossover rate 1 (alpha <= p_c always) every
    offspring equals its parent, so generations change nothing; recipes stay inside [lo, hi]; only the
    current group's coordinates differ from the best-so-far in any evaluated recipe."""
    from oracle.recipe_search import search_recipe
    center = [0.9, 0.2, 0.5, 0.7, 0.95, 0.1, 0.33]
    seen = []

    def loss(rho):
        seen.append(list(rho))
        return _quad(center)(rho)

    S, best, hist = search_recipe(loss, 7, population=12, generations=6, group_size=3, seed=5, lo=0.05, hi=0.98)
    assert all(b <= a for a, b in zip(hist, hist[1:])) and best == hist[-1] == _quad(center)(S)
    assert len(hist) == 1 + 3 * 6 and best < hist[0]
    assert all(0.05 <= v <= 0.98 for rho in seen for v in rho)
    # group structure: evaluations of group g differ from the first evaluation (the start) only in groups <= g
    n_eval_group = 11 + 6 * 12
    for gi, (lo_c, hi_c) in enumerate(((0, 3), (3, 6), (6, 7))):
        block = seen[1 + gi * n_eval_group: 1 + (gi + 1) * n_eval_group]
        ref = block[0]
        for rho in block:
            outside = [c for c in range(7) if not lo_c <= c < hi_c]
            assert all(rho[c] == ref[c] for c in outside)
    S0, best0, hist0 = search_recipe(_quad(center), 7, population=12, generations=0, group_size=7, seed=5)
    assert len(hist0) == 1
    S1, best1, hist1 = search_recipe(_quad(center), 7, population=12, generations=4, p_c=1.0, group_size=7, seed=5)
    assert hist1[1:] == [hist1[1]] * 4 and best1 == hist1[1]
    # reproducible, and the seed matters
    assert search_recipe(_quad(center), 7, seed=9)[0] == search_recipe(_quad(center), 7, seed=9)[0]
    assert search_recipe(_quad(center), 7, seed=9)[0] != search_recipe(_quad(center), 7, seed=10)[0]


def test_recipe_search_finds_the_minimiser_of_a_separable_loss():
    """With the paper's settings (population 32, 5 generations, p_m = p_c = 0.5) but more generations,
    the search closes in on the known minimiser of a convex separable loss, coordinate by coordinate."""
    from oracle.recipe_search import search_recipe
    rng = np.random.default_rng(2)
    center = rng.uniform(0.1, 0.9, 12).tolist()
    S, best, hist = search_recipe(_quad(center), 12, population=32, generations=40, group_size=4, seed=1)
    assert best < 1e-3 * hist[0]
    assert np.max(np.abs(np.array(S) - np.array(center))) < 0.02
    # a start that is already optimal is kept
    S2, best2, _ = search_recipe(_quad(center), 12, population=8, generations=3, group_size=4, seed=1, rho_start=center)
    assert best2 == 0.0 and S2 == center


def test_recipe_search_uniform_stream():
    """The random stream: splitmix64 outputs for seed 0 are the published reference values; the
    uniforms lie in [0, 1) with the right mean."""
    from oracle.recipe_search import _splitmix64, _Uniform
    assert _splitmix64(0, 0) == 0xE220A8397B1DCDAF and _splitmix64(0, 1) == 0x6E789E6AA1B965F4
    u = _Uniform(123)
    xs = np.array([u() for _ in range(20000)])
    assert xs.min() >= 0.0 and xs.max() < 1.0 and abs(xs.mean() - 0.5) < 0.01


# --------------------------------------------------------------------------- 4-bit weights (Sec. 4.4)

def test_q4_hand_worked_golden():
    """Dequantisation and the layer on it, against numbers worked by hand from the format's definition."""
    path = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_q4.txt")
    item = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#") or line.startswith("case:"):
                continue
            key, val = line.split(":", 1)
            item[key.strip()] = [[float(v) for v in row.split()] for row in val.split(";")]
    group = int(item["group"][0][0])
    Q = np.array(item["Q"], dtype=np.uint8)
    Z = np.array(item["Z"], dtype=np.uint8)
    for dt in (oracle.F16, oracle.BF16):
        S16 = synth.encode16(np.array(item["S"]), dt)
        assert oracle.dequant_q4(Q, S16, Z, dt, group).tolist() == item["expect W"]
        X16 = synth.encode16(np.array(item["X"]), dt)
        tau = item["tau"][0][0]
        out0 = oracle.rsparse_linear_q4(Q, S16, Z, None, None, X16, dt, tau, group=group)
        assert out0["act"][0].tolist() == [int(v) for v in item["expect rank=0 kept"][0]]
        assert out0["Y"].tolist() == item["expect rank=0 Y"]
        U16 = synth.encode16(np.array(item["U"]), dt)
        SV16 = synth.encode16(np.array(item["SV"]), dt)
        out1 = oracle.rsparse_linear_q4(Q, S16, Z, U16, SV16, X16, dt, tau, group=group)
        assert out1["Y"].tolist() == item["expect rank=1 Y"]


def test_q4_single_code_lands_on_its_own_row_channel_and_group():
    """One non-zero (q - z) at a time: the value must appear at exactly [o][c] with the scale of group
    c / group of row o -- a transposed operand or a group taken along the wrong axis fails here."""
    d_out, d_in, group = 3, 8, 4
    G = d_in // group
    scales = np.array([[1.0, 2.0], [4.0, 8.0], [16.0, 32.0]])
    S16 = synth.encode16(scales, oracle.F16)
    Z = np.full((d_out, G), 5, dtype=np.uint8)
    for o in range(d_out):
        for c in range(d_in):
            Q = np.full((d_out, d_in), 5, dtype=np.uint8)
            Q[o, c] = 7
            W = oracle.dequant_q4(Q, S16, Z, oracle.F16, group)
            want = np.zeros((d_out, d_in))
            want[o, c] = 2.0 * scales[o, c // group]
            assert np.array_equal(W, want), (o, c)


def test_q4_grid_round_trip_and_rounding_bound():
    """Two properties that tie the oracle's dequantisation to the (independent) synthetic quantiser.
    Weights built on a known grid (power-of-two scale, codes 0 and 15 present in every group) are
    recovered exactly, codes included; arbitrary weights come back within half a step of the stored
    scale, plus what the 16-bit rounding of the scale can shift the top of the range."""
    rng = np.random.default_rng(11)
    d_out, d_in, group = 16, 256, 128
    G = d_in // group
    for dt in (oracle.F16, oracle.BF16):
        s_true = 2.0 ** rng.integers(-9, -3, size=(d_out, G)).astype(np.float64)
        z_true = rng.integers(0, 16, size=(d_out, G))
        q_true = rng.integers(0, 16, size=(d_out, d_in))
        q_true[:, 0::group] = 0
        q_true[:, 1::group] = 15
        W = np.repeat(s_true, group, axis=1) * (q_true - np.repeat(z_true, group, axis=1))
        Q, S16, Z = synth.quantize_q4(W, dt, group)
        assert np.array_equal(Q, q_true) and np.array_equal(Z, z_true)
        assert np.array_equal(oracle.dequant_q4(Q, S16, Z, dt, group), W)

        W = rng.standard_normal((d_out, d_in)) * 0.02
        Q, S16, Z = synth.quantize_q4(W, dt, group)
        assert Q.max() <= 15 and Z.max() <= 15
        Wq = oracle.dequant_q4(Q, S16, Z, dt, group)
        s = np.repeat(synth.decode16(S16, dt), group, axis=1)
        eps = 2.0 ** (-8 if dt == oracle.BF16 else -11)
        assert np.all(np.abs(W - Wq) <= 0.5 * s + 16.0 * s * eps + 0.5 * s)   # zero-point rounding: another half step
        assert np.mean(np.abs(W - Wq) <= 0.5 * s * (1 + 1e-12)) > 0.9


def test_q4_all_channels_kept_is_the_dense_product_with_the_dequantised_weights():
    rng = np.random.default_rng(5)
    d_out, d_in, group = 24, 256, 128
    W = rng.standard_normal((d_out, d_in)) * 0.05
    Q, S16, Z = synth.quantize_q4(W, oracle.BF16, group)
    X16 = synth.encode16(rng.standard_normal((2, d_in)), oracle.BF16)
    out = oracle.rsparse_linear_q4(Q, S16, Z, None, None, X16, oracle.BF16, -math.inf, group=group)
    Wq = oracle.dequant_q4(Q, S16, Z, oracle.BF16, group)
    want = oracle.dense_linear(Wq, X16, oracle.F64, oracle.BF16)
    assert np.array_equal(out["Y"], want)
    # and the dequantised matrix is what numpy's integer arithmetic gives
    s = np.repeat(synth.decode16(S16, oracle.BF16), group, axis=1)
    z = np.repeat(Z.astype(np.int64), group, axis=1)
    assert np.array_equal(Wq, s * (Q.astype(np.int64) - z))


def test_q4_rejects_codes_out_of_range():
    Q = np.zeros((1, 4), dtype=np.uint8)
    Q[0, 1] = 16
    S16 = synth.encode16(np.ones((1, 2)), oracle.F16)
    Z = np.zeros((1, 2), dtype=np.uint8)
    with pytest.raises(ValueError):
        oracle.dequant_q4(Q, S16, Z, oracle.F16, 2)
