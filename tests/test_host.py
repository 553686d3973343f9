"""CPU-only checks of the product's host code: the C ABI loads and exports every declared symbol,
argument validation, threshold calibration against the oracle, the byte model, the host SVD."""
import math
import os
import re

import numpy as np
import pytest

import oracle
import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "rsparse.h")).read()
    declared = sorted(set(re.findall(r"\b(rsparse_[a-z0-9_]+)\s*\(", header)))
    lib = rs.load_library()
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in rsparse.h but not exported"
    assert sorted(rs.EXPORTED_SYMBOLS) == declared


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_19449_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                for pat in (r"^\s*(import|from)\s+oracle", r"librsparse_oracle", r"\borc_[a-z]", r"rsparse_oracle"):
                    assert not re.search(pat, text, re.M), f"{f} reaches into the oracle ({pat})"


@pytest.mark.parametrize("bad", [
    dict(d_in=12), dict(d_out=0), dict(rank=-1), dict(rank=72), dict(rank=12), dict(max_batch=0), dict(max_batch=33),
    dict(tau=float("nan")), dict(dtype=2), dict(out_dtype=0, dtype=1), dict(cmp_mode=3), dict(batch_mask_mode=-1),
    dict(batch_mask_mode=3), dict(lowrank_channel_major=2), dict(lowrank_channel_major=-1), dict(topk=-1), dict(topk=65), dict(topk=8, cmp_mode=1), dict(topk=8, cmp_mode=2),
])
def test_config_validation(bad):
    kw = dict(d_in=64, d_out=64, rank=8, tau=0.5, dtype=rs.F16, max_batch=1)
    kw.update(bad)
    cfg = rs.make_config(kw["d_in"], kw["d_out"], kw["rank"], kw["tau"], kw["dtype"], max_batch=kw["max_batch"],
                         out_dtype=kw.get("out_dtype"), cmp_mode=kw.get("cmp_mode", 0),
                         batch_mask_mode=kw.get("batch_mask_mode", 0), topk=kw.get("topk", 0),
                         lowrank_channel_major=kw.get("lowrank_channel_major", 0))
    W = np.zeros((max(kw["d_out"], 1), max(kw["d_in"], 1)), dtype=np.uint16)
    lib = rs.load_library()
    import ctypes as C
    h = C.c_void_p()
    st = lib.rsparse_prepare_factors(C.byref(cfg), W.ctypes.data_as(C.c_void_p), None, None, C.byref(h))
    assert st == 1 and h.value is None
    assert rs.rsparse_last_error()


def test_null_arguments_are_rejected():
    import ctypes as C
    lib = rs.load_library()
    assert lib.rsparse_linear(None, None, 1, None, None) == 1
    assert lib.rsparse_dense_ref(None, None, 1, None, None) == 1
    assert lib.rsparse_linear_group(None, 1, None, 1, None, None) == 1
    assert lib.rsparse_dense_ref_group(None, 0, None, 1, None, None) == 1
    assert lib.rsparse_last_active(None, 0, None, None) == 1
    assert lib.rsparse_set_tau(None, 0.5) == 1
    assert lib.rsparse_calibrate_tau(None, 0, 10, 0.5, None) == 1
    assert lib.rsparse_required_bytes(None, 1, 1) == 0
    lib.rsparse_destroy(None)


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("s", [0.0, 0.4, 0.5, 0.7, 1.0])
def test_calibrate_tau_matches_the_oracle_bit_for_bit(dt, s):
    src = synth.DModelInput(512, config=70, linear=dt)
    X16 = synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), dt)
    got = rs.rsparse_calibrate_tau(X16, dt, s)
    want = oracle.quantile_tau(X16, dt, s)
    assert got == want


def test_compute_factors_weyl_and_eckart_young():
    """Host SVD on W = U diag(sigma) V^T (rounded to 16 bit): singular values within ||E||_2 of the
    closed form (Weyl), and the rank-r product attains the Eckart-Young error sum_{i>r} sigma_i^2.
    A spectrum with a gap after r makes the truncation well conditioned."""
    d_in, d_out, r = 192, 128, 24
    p = min(d_in, d_out)
    sigma = np.concatenate([np.linspace(2.0, 1.0, r), 0.3 * np.arange(1, p - r + 1) ** -0.6])
    L = synth.make_layer(d_in, d_out, r, synth.BF16, config=71, linear=0, sigma=sigma)
    cfg = rs.make_config(d_in, d_out, r, 0.5, synth.BF16)
    U16, SV16, sig = rs.rsparse_compute_factors(cfg, L.W16)
    Wd = synth.decode16(L.W16, L.dtype)
    E = Wd - (L.U * L.sigma) @ L.V.T
    assert np.max(np.abs(sig - sigma[:r])) <= np.linalg.norm(E, 2) * 1.01
    s_true = np.linalg.svd(Wd, compute_uv=False)
    assert np.allclose(sig, s_true[:r], rtol=1e-8)
    approx = synth.decode16(U16, L.dtype) @ synth.decode16(SV16, L.dtype)
    tail = np.sum(s_true[r:] ** 2)
    err = np.linalg.norm(Wd - approx) ** 2
    # the stored factors are rounded to bf16 (relative 2^-9 each): allow that on top of the optimum
    slack = (2 * 2.0 ** -9) ** 2 * np.sum(s_true[:r] ** 2)
    assert tail * (1 - 1e-9) <= err <= tail + 4 * slack
    # U_r has orthonormal columns up to storage rounding
    Ud = synth.decode16(U16, L.dtype)
    assert np.max(np.abs(Ud.T @ Ud - np.eye(r))) < 0.02


def test_compute_factors_power_law_spectrum_fp16():
    L = synth.make_layer(160, 224, 16, synth.F16, config=71, linear=1)
    cfg = rs.make_config(160, 224, 16, 0.5, synth.F16)
    U16, SV16, sig = rs.rsparse_compute_factors(cfg, L.W16)
    Wd = synth.decode16(L.W16, L.dtype)
    s_true = np.linalg.svd(Wd, compute_uv=False)
    assert np.allclose(sig, s_true[:16], rtol=1e-7)
    approx = synth.decode16(U16, L.dtype) @ synth.decode16(SV16, L.dtype)
    tail = np.sum(s_true[16:] ** 2)
    assert np.linalg.norm(Wd - approx) ** 2 <= tail * 1.01 + 1e-6


def test_recipe_mapping_of_sec_3_5():
    """s = rho C, r = (1 - rho) C mn / (m + n).  The uniform recipe the paper uses (rho = 0.95) at a 50 %
    budget gives s = 0.475 and r = 0.025 * mn/(m+n): 51.2 for 4096x4096, 74.6 for 4096x11008; the library
    rounds r down to its granularity of 8.  The relative I/O of the result follows the cost model of
    Sec. 3.4, r (m + n) / (mn) + s, and never exceeds the budget."""
    s, r, io = rs.rsparse_recipe(4096, 4096, 0.5, 0.95)
    assert s == pytest.approx(0.475) and r == 48 and 0.025 * 4096 * 4096 / 8192 == pytest.approx(51.2)
    assert io == pytest.approx(48 * 8192 / 4096 ** 2 + 0.475) and io <= 0.5
    s, r, io = rs.rsparse_recipe(4096, 11008, 0.5, 0.95)
    assert r == 72 and 0.025 * 4096 * 11008 / (4096 + 11008) == pytest.approx(74.63, abs=0.01) and io <= 0.5
    assert rs.rsparse_recipe(4096, 4096, 0.5, 1.0)[:2] == (0.5, 0)            # "Sparse" baseline of Sec. 4.4
    s, r, io = rs.rsparse_recipe(4096, 4096, 0.5, 0.0)                        # "Low-Rank" baseline
    assert s == 0.0 and r == 1024 and io == pytest.approx(0.5)
    assert rs.rsparse_recipe(64, 64, 1.0, 0.0)[1] == 32                       # mn/(m+n) = 32 <= min(m, n)
    for bad in ((0, 8, 0.5, 0.5), (8, 8, 1.5, 0.5), (8, 8, 0.5, -0.1), (8, 8, float("nan"), 0.5)):
        with pytest.raises(rs.RSparseError):
            rs.rsparse_recipe(*bad)


def test_recipe_search_matches_the_oracle_bit_for_bit():
    """rsparse_search_recipe (host C++) against the plain-Python oracle of Sec. 3.5's algorithm: same
    seed, same loss => the same recipe, best loss and per-generation history, exactly."""
    from oracle.recipe_search import search_recipe
    rng = np.random.default_rng(4)
    for L, P, T, gs, seed, pm, pc in ((5, 8, 3, 2, 1, 0.5, 0.5), (30, 32, 5, 28, 7, 0.5, 0.5), (9, 6, 4, 9, 11, 0.8, 0.3)):
        center = rng.uniform(0.0, 1.0, L)
        w = rng.uniform(0.5, 2.0, L)

        def loss(rho):
            return float(np.sum(w * (np.asarray(rho) - center) ** 2) + 0.1 * np.sin(7.0 * np.sum(rho)))

        want = search_recipe(loss, L, population=P, generations=T, p_m=pm, p_c=pc, group_size=gs, seed=seed, lo=0.02, hi=0.99)
        got = rs.rsparse_search_recipe(loss, L, population=P, generations=T, p_m=pm, p_c=pc, group_size=gs, seed=seed,
                                       lo=0.02, hi=0.99)
        assert got[0].tolist() == want[0] and got[1] == want[1] and got[2].tolist() == want[2]
    start = [0.3, 0.6, 0.9]
    want = search_recipe(lambda r: abs(r[0] - 0.5) + r[1] * r[2], 3, population=4, generations=2, group_size=1, seed=3, rho_start=start)
    got = rs.rsparse_search_recipe(lambda r: abs(r[0] - 0.5) + r[1] * r[2], 3, population=4, generations=2, group_size=1, seed=3,
                                   rho_start=start)
    assert got[0].tolist() == want[0] and got[2].tolist() == want[2]
    with pytest.raises(rs.RSparseError):
        rs.rsparse_search_recipe(lambda r: 0.0, 0)


@pytest.mark.parametrize("bad", [
    dict(group=48), dict(group=16), dict(group=2048), dict(group=256, d_in=384), dict(max_batch=33),
    dict(code=16), dict(zero=16), dict(null="Q"), dict(null="S"), dict(null="Z"),
])
def test_q4_argument_validation(bad):
    """Every check of rsparse_prepare_q4 happens before the first device call, so it is testable here."""
    import ctypes as C
    d_in, d_out, group = bad.get("d_in", 256), 16, bad.get("group", 128)
    cfg = rs.make_config(d_in, d_out, 0, 0.5, rs.F16, max_batch=bad.get("max_batch", 1),
                         dense_rowmajor=bad.get("dense_rowmajor", 0))
    G = max(1, d_in // group)
    Q = np.zeros((d_out, d_in), dtype=np.uint8)
    S = np.zeros((d_out, G), dtype=np.uint16)
    Z = np.zeros((d_out, G), dtype=np.uint8)
    if "code" in bad:
        Q[3, 5] = bad["code"]
    if "zero" in bad:
        Z[2, 0] = bad["zero"]
    ptr = {k: v.ctypes.data_as(C.c_void_p) for k, v in (("Q", Q), ("S", S), ("Z", Z))}
    if "null" in bad:
        ptr[bad["null"]] = None
    h = C.c_void_p()
    st = rs.load_library().rsparse_prepare_q4(C.byref(cfg), ptr["Q"], ptr["S"], ptr["Z"], group, None, None, C.byref(h))
    assert st == 1 and h.value is None
    assert rs.rsparse_last_error()


def test_plan_layer_byte_model_and_decisions():
    """rsparse_plan_layer: the estimate is Sec. 3.4's byte model over a fixed rate plus a fixed cost per launch,
    so it must be monotone in everything that adds bytes, and must reproduce the clear-cut decisions: small
    attention projections dense, the large MLP layers with R-Sparse, nothing with R-Sparse when every channel
    is kept."""
    rs_small, d_small, use_small = rs.rsparse_plan_layer(4096, 4096, 256, 0.5)
    assert not use_small and rs_small > d_small
    rs_big, d_big, use_big = rs.rsparse_plan_layer(8192, 28672, 1024, 0.5)
    assert use_big and 1.2 < d_big / rs_big < 1.6
    assert not rs.rsparse_plan_layer(8192, 28672, 1024, 1.0)[2]
    # exact arithmetic of the model on one case: bytes / 6.5e6 + fixed / group
    us_rs, us_d, _ = rs.rsparse_plan_layer(4096, 11008, 512, 0.5, group=2)
    io = 2.0 * (4096 + 11008)
    want_rs = 8.5 / 2 + (2.0 * (0.5 * 4096 * 11008 + 512 * (4096 + 11008)) + io) / 6.5e6
    want_d = 3.6 / 2 + (2.0 * 4096 * 11008 + io) / 6.5e6
    assert abs(us_rs - want_rs) < 1e-9 and abs(us_d - want_d) < 1e-9
    # monotone: more kept channels and more rank never make R-Sparse cheaper; sharing a launch never dearer
    base = rs.rsparse_plan_layer(4096, 11008, 256, 0.4)[0]
    assert rs.rsparse_plan_layer(4096, 11008, 256, 0.6)[0] > base
    assert rs.rsparse_plan_layer(4096, 11008, 512, 0.4)[0] > base
    assert rs.rsparse_plan_layer(4096, 11008, 256, 0.4, group=2)[0] < base
    # more than one token: the union of the kept channels grows as 1 - (1 - s)^B, the matrix-core path reads all of W:
    # the 70B-shape MLP layers still pay at 2 tokens, nothing pays from 8 tokens on
    assert rs.rsparse_plan_layer(8192, 28672, 1024, 0.5, 2, 2)[2]
    for B in (8, 16, 32):
        for shape in ((4096, 4096, 256), (8192, 28672, 1024), (28672, 8192, 1024)):
            est_rs, est_d, use = rs.rsparse_plan_layer(*shape, 0.5, 1, B)
            assert not use and est_rs > est_d
    b2 = rs.rsparse_plan_layer(4096, 11008, 512, 0.5, 1, 2)
    u2 = 1 - 0.5 ** 2
    want2 = (8.5 + 3.0) + (2.0 * (u2 * 4096 * 11008 + 512 * (4096 + 11008)) + 2.0 * 2 * (4096 + 11008)) / 6.7e6
    assert abs(b2[0] - want2) < 1e-9
    for bad in (dict(d_in=0), dict(rank=5000), dict(keep_fraction=1.5), dict(group=0), dict(group=5), dict(batch=0), dict(batch=33)):
        kw = dict(d_in=4096, d_out=4096, rank=256, keep_fraction=0.5, group=1)
        kw.update(bad)
        with pytest.raises(rs.RSparseError):
            rs.rsparse_plan_layer(**kw)


def test_io_model_is_the_byte_form_of_sec_3_4():
    """rsparse_io_model (which rsparse_required_bytes / rsparse_dense_bytes evaluate for a handle) against
    the paper's own cost model: relative memory I/O r (m + n) / (m n) + s with s the share of columns loaded
    (Sec. 3.4), here in bytes with the token and the output added, for every benchmark shape; byte counts
    worked out by hand for the 4096 x 4096 and the 4096 / 11008 shapes are reproduced to the byte."""
    shapes = [(4096, 4096, 256, rs.F16), (4096, 11008, 512, rs.BF16), (11008, 4096, 512, rs.BF16),
              (4096, 14336, 256, rs.BF16), (4096, 1024, 128, rs.BF16), (8192, 28672, 1024, rs.BF16),
              (28672, 8192, 1024, rs.BF16), (8192, 1024, 1024, rs.BF16), (1032, 1096, 40, rs.F16)]
    for d_in, d_out, r, dt in shapes:
        for B in (1, 2, 8, 32):
            for k in (0, d_in // 2, (d_in * 3) // 10, d_in):
                for out in (dt, rs.F32):
                    cfg = rs.make_config(d_in, d_out, r, 0.0, dt, max_batch=32, out_dtype=out)
                    req, dense, req_in = rs.rsparse_io_model(cfg, B, k)
                    eo = 4 if out == rs.F32 else 2
                    io = 2 * B * d_in + eo * B * d_out
                    assert dense == 2 * d_in * d_out + io
                    assert req == 2 * (k * d_out + r * d_out + r * d_in) + io
                    assert req_in == 2 * (k * d_out + r * d_out + r * (d_in - k)) + io
                    # the paper's relative form: (required - token - output) / W bytes = r (m + n) / (m n) + s
                    m, n, s = d_out, d_in, k / d_in
                    assert math.isclose((req - io) / (2 * d_in * d_out), r * (m + n) / (m * n) + s, rel_tol=1e-12)
    # tabulated values: 4096 x 4096, r = 256, half the channels -> 20.99 MB against 33.57 MB (ratio 0.625);
    # 4096 -> 11008, r = 512: 60.59 MB against 90.21 MB
    req, dense, req_in = rs.rsparse_io_model(rs.make_config(4096, 4096, 256, 0.0, rs.F16), 1, 2048)
    assert (req, dense) == (20987904, 33570816) and abs(req / dense - 0.625) < 3e-4
    assert abs(dense / req_in - 1.68) < 0.005
    req, dense, _ = rs.rsparse_io_model(rs.make_config(4096, 11008, 512, 0.0, rs.BF16), 1, 2048)
    assert round(req / 1e6, 2) == 60.59 and round(dense / 1e6, 2) == 90.21
    # 4-bit weights, groups of 128: half a byte per weight, 2.5 bytes per output and touched group
    cfg = rs.make_config(4096, 11008, 512, 0.0, rs.BF16)
    req, dense, _ = rs.rsparse_io_model(cfg, 1, 2048, q4_group=128)
    fac = 2 * (512 * 11008 + 512 * 4096)
    assert dense == 4096 * 11008 // 2 + 32 * 11008 * 5 // 2 + 2 * 4096 + 2 * 11008
    assert req == 2048 * 11008 // 2 + 32 * 11008 * 5 // 2 + fac + 2 * 4096 + 2 * 11008
    assert rs.rsparse_io_model(cfg, 1, 3, q4_group=128)[0] == 3 * 11008 // 2 + 3 * 11008 * 5 // 2 + fac + 2 * 4096 + 2 * 11008
    for bad in (dict(batch=0), dict(batch=33), dict(k_union=-1), dict(k_union=4097), dict(q4_group=100), dict(q4_group=16)):
        kw = dict(batch=1, k_union=10, q4_group=0)
        kw.update(bad)
        with pytest.raises(rs.RSparseError):
            rs.rsparse_io_model(cfg, **kw)


def test_bf16_encodings_round_fp64_once():
    """The generator's bf16 encoder and the library's factor rounding (through rsparse_compute_factors' stored
    factors) round a double ONCE: equal to the oracle's rounding-by-definition, also on doubles that a detour
    through fp32 would first push onto a tie."""
    rng = np.random.default_rng(17)
    v = rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))
    base = synth.decode16(rng.integers(0x0080, 0x7F00, 50000).astype(np.uint16), synth.BF16)      # bf16 values
    nxt = synth.decode16((synth.encode16(base, synth.BF16).astype(np.uint32) + 1).astype(np.uint16), synth.BF16)
    mid = 0.5 * (base + nxt)                                                                       # exact ties
    near = np.concatenate([mid * (1 + 2.0 ** -40), mid * (1 - 2.0 ** -40), mid, -mid * (1 + 2.0 ** -45)])
    allv = np.concatenate([v, near, [0.0, -0.0, np.inf, -np.inf, 1e39, -1e39, 1e-45]])
    assert np.array_equal(synth.encode16(allv, synth.BF16), oracle.round16_from_double(allv, synth.BF16))
    assert np.array_equal(synth.encode16(allv, synth.F16), oracle.round16_from_double(allv, synth.F16))


def test_multiphase_bias_is_the_mean_residual_of_sec_3_2():
    """Host routine against the oracle's literal form (per token: interval sets, column sums, midpoints; then the mean)."""
    import oracle
    g = np.random.Generator(np.random.PCG64(77))
    for dt in (synth.F16, synth.BF16):
        d_in, d_out, N = 96, 40, 7
        W16 = synth.encode16(g.standard_normal((d_out, d_in)) * 0.2, dt)
        H16 = synth.encode16(g.standard_normal((N, d_in)), dt)
        H16[0, :4] = synth.encode16(np.array([0.5, -0.25, -3.0, np.nan]), dt)        # ties at every threshold, a NaN
        for T in ([0.5], [0.5, -0.25], [0.5, -0.25, -3.0], [1.0, 0.0, -1.0, -2.0]):
            got = rs.rsparse_multiphase_bias(W16, dt, H16, T)
            Hc = H16.copy()
            nan = np.isnan(synth.decode16(Hc, dt))
            want = oracle.static_bias(W16, dt, Hc, dt, np.array(T, dtype=np.float64))
            assert not np.any(np.isnan(got))
            assert np.allclose(got, want, rtol=2e-6, atol=1e-7), T                   # one rounding to fp32
            assert nan.sum() == 1
    lib = rs.load_library()
    import ctypes as C
    out = np.zeros(8, dtype=np.float32)
    W = np.zeros((8, 8), dtype=np.uint16)
    bad_T = np.array([0.0, 0.0], dtype=np.float32)
    st = lib.rsparse_multiphase_bias(W.ctypes.data_as(C.c_void_p), 0, 8, 8, W.ctypes.data_as(C.c_void_p), 1,
                                     bad_T.ctypes.data_as(C.c_void_p), 2, out.ctypes.data_as(C.c_void_p))
    assert st == 1
