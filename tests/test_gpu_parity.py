"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Kept-channel lists must be equal; outputs within the stated tolerances."""
import numpy as np
import pytest

import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
INF = float("inf")


@pytest.fixture(scope="module")
def ragged():
    """Several column tiles with a ragged tail (1096 = 2*512 + 72), d_in not a multiple of 256."""
    return {dt: synth.make_layer(1032, 1096, 40, dt, config=81, linear=dt) for dt in (synth.F16, synth.BF16)}


@pytest.fixture(scope="module")
def config0():
    return synth.make_layer(4096, 4096, 256, synth.F16, config=0, linear=0)


def _parity(L, X16, tau, out_dtype=None, max_batch=None, tuning=None, **cfg_kw):
    X16 = np.atleast_2d(X16)
    layer = gu.prepare(L, tau, max_batch=max_batch or X16.shape[0], out_dtype=out_dtype, **cfg_kw)
    if tuning:
        rs.rsparse_set_tuning(layer, **tuning)
    got = gu.run_linear(layer, X16)
    want = gu.oracle_linear(L, X16, tau, cmp_mode=cfg_kw.get("cmp_mode", 0),
                            batch_mask_mode=cfg_kw.get("batch_mask_mode", 0))
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
    layer.destroy()
    return got, want


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("out", [None, rs.F32])
def test_ragged_batch1(ragged, dt, out):
    L = ragged[dt]
    X16, src = gu.tokens_for(L, 3, linear=dt)
    tau = gu.calibrated_tau(L, src, 0.5)
    for b in range(3):
        got, _ = _parity(L, X16[b], tau, out_dtype=out)
        assert 0.3 * L.d_in < len(got["act"][0]) < 0.7 * L.d_in


@pytest.mark.parametrize("out", [None, rs.F32])
def test_config0_full_size(config0, out):
    """configs[0]: 4096x4096 fp16, r = 256, tau = 50% quantile of 64 calibration tokens."""
    L = config0
    src = synth.DModelInput(L.d_in, config=0, linear=0)
    tau = gu.calibrated_tau(L, src, 0.5)
    X16 = synth.encode16(src.tokens(4), L.dtype)
    for b in range(4):
        got, _ = _parity(L, X16[b], tau, out_dtype=out)
        assert abs(len(got["act"][0]) - 2048) < 200


def test_edge_thresholds(ragged):
    L = ragged[synth.F16]
    X16, _ = gu.tokens_for(L, 1)
    for tau in (-INF, 0.0, INF, 1e30):
        for mode in (0, 1):
            _parity(L, X16, tau, out_dtype=rs.F32, cmp_mode=mode)


def test_all_ties_token(ragged):
    L = ragged[synth.BF16]
    x = np.where(np.arange(L.d_in) % 3 == 0, -0.75, 0.75)
    X16 = synth.encode16(x, L.dtype)
    got0, _ = _parity(L, X16, 0.75, cmp_mode=0)
    got1, _ = _parity(L, X16, 0.75, cmp_mode=1)
    assert len(got0["act"][0]) == L.d_in and len(got1["act"][0]) == 0


def test_rank_zero_and_full_rank():
    L0 = synth.make_layer(520, 264, 0, synth.F16, config=82, linear=0)
    X16, src = gu.tokens_for(L0, 2)
    tau = gu.calibrated_tau(L0, src, 0.6)
    _parity(L0, X16[0], tau, out_dtype=rs.F32)
    Lf = synth.make_layer(520, 264, 264, synth.F16, config=82, linear=0)
    got, _ = _parity(Lf, X16[1], tau, out_dtype=rs.F32)
    # full rank: the layer is (up to factor rounding) the dense product
    dense = synth.decode16(X16[1], Lf.dtype) @ synth.decode16(Lf.W16, Lf.dtype).T
    assert np.linalg.norm(got["Y"][0] - dense) <= 5e-3 * np.linalg.norm(dense)


def test_nan_inf_inputs(ragged):
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 1)
    tau = gu.calibrated_tau(L, src, 0.5)
    X = X16[0].copy()
    X[5] = 0x7C00          # +inf: kept
    X[77] = 0xFC00         # -inf: kept
    X[8] = 0x8000          # -0
    got, want = _parity(L, X, tau, out_dtype=rs.F32)
    assert 5 in got["act"][0] and 77 in got["act"][0] and 8 not in got["act"][0]
    X[9] = 0x7E00          # NaN: never kept, goes through the low-rank path and poisons the output
    got, want = _parity(L, X, tau, out_dtype=rs.F32)
    assert 9 not in got["act"][0]
    assert np.all(np.isnan(got["Y"]))


def test_fp16_subnormal_weights_are_not_flushed():
    L = synth.make_layer(264, 520, 8, synth.F16, config=83, linear=0)
    W = synth.decode16(L.W16, L.dtype)
    scale = 3e-5 / np.max(np.abs(W))           # push every weight into fp16's subnormal range
    L.W16 = synth.encode16(W * scale, L.dtype)
    assert np.all((L.W16 & 0x7C00) == 0) and np.count_nonzero(L.W16 & 0x3FF) > 0.9 * L.W16.size
    L.rank, L.U16, L.SV16 = 0, L.U16[:, :0], L.SV16[:0]
    X16, _ = gu.tokens_for(L, 1)
    got, want = _parity(L, X16, 0.5, out_dtype=rs.F32)
    assert np.linalg.norm(want["Y"]) > 0


@pytest.mark.parametrize("B", [2, 3, 4, 5, 8, 9, 16, 32])
@pytest.mark.parametrize("mask_mode", [0, 1])
def test_batches(ragged, B, mask_mode):
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, B, linear=B)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16, tau, out_dtype=rs.F32, batch_mask_mode=mask_mode)
    _parity(L, X16, tau, batch_mask_mode=mask_mode)


def test_batch_smaller_than_max_batch_and_reuse(ragged):
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 8)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=8, out_dtype=rs.F32)
    for B in (8, 1, 3, 8, 2):
        got = gu.run_linear(layer, X16[:B])
        want = gu.oracle_linear(L, X16[:B], tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    # tau sweep without re-packing
    for s in (0.4, 0.7):
        t2 = gu.calibrated_tau(L, src, s)
        rs.rsparse_set_tau(layer, t2)
        got = gu.run_linear(layer, X16[:2])
        want = gu.oracle_linear(L, X16[:2], t2)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
        assert abs(len(got["act"][0]) / L.d_in - (1 - s)) < 0.1


@pytest.mark.parametrize("tuning", [
    dict(splits=1), dict(splits=3, waves=1), dict(splits=7, waves=2), dict(splits=64, waves=8),
    dict(splits=500, waves=4), dict(lowrank_rows=2), dict(lowrank_rows=4, nontemporal=1),
    dict(launches=2), dict(launches=2, splits=7, waves=2), dict(launches=2, lowrank_rows=4, nontemporal=1),
])
def test_launch_shapes(ragged, tuning):
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 4)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16[0], tau, out_dtype=rs.F32, tuning=tuning)
    _parity(L, X16, tau, out_dtype=rs.F32, tuning=tuning)


@pytest.mark.parametrize("launches", [1, 2])
@pytest.mark.parametrize("B", [1, 3, 8, 12])
def test_one_and_two_launch_forms_on_a_reused_handle(ragged, launches, B):
    """Both forms of the vector path (stage 2 inside the gather launch, or in a second kernel), called
    back to back on one handle with different kept sets: the arrival counters and accumulators of the
    one-launch form must be back at zero after every call.  12 tokens = two batch tiles."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, B, linear=40 + B)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=B, out_dtype=rs.F32)
    rs.rsparse_set_tuning(layer, launches=launches, mfma_min_batch=33)
    for t in (tau, -INF, gu.calibrated_tau(L, src, 0.7), INF, tau):
        rs.rsparse_set_tau(layer, t)
        got = gu.run_linear(layer, X16)
        rs.rsparse_synchronize(layer)
        want = gu.oracle_linear(L, X16, t)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_gated_input_bits_equal_the_oracle_for_every_gate_value(dt):
    """rsparse_gated_input against the oracle's own copy of the recipe, bit for bit: all 65 536 gate
    patterns (NaNs compared as NaN) times up-values that reach subnormals, overflow, zero, Inf."""
    import oracle
    torch = gu.torch_mod()
    ups = synth.encode16(np.array([1.0, -0.37, 3.1, 1e-4, 250.0, 7e-3, 0.11, -33.0, 0.0, -0.0, 6e4, -2e-7,
                                   np.inf, 1.0009765625, -7.5, 2e-3]), dt)
    G = np.repeat(np.arange(65536, dtype=np.uint16), len(ups))
    U = np.tile(ups, 65536)
    want = oracle.gated_input(G, U, dt)
    Gd, Ud = gu.to_dev16(G), gu.to_dev16(U)
    out = torch.zeros_like(Gd)
    rs.rsparse_gated_input(Gd.data_ptr(), Ud.data_ptr(), out.data_ptr(), G.size, dt, gu.stream_ptr())
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    both_nan = np.isnan(synth.decode16(got, dt)) & np.isnan(synth.decode16(want, dt))
    assert np.array_equal(got[~both_nan], want[~both_nan])
    assert both_nan.sum() >= 2 * 1000


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_gated_input_against_the_plain_definition(dt):
    """rsparse_gated_input against the plain definition of Sec. 3.1's activation, u * g / (1 + exp(-g)) in
    fp64 with one rounding to 16 bits (no recipe on the oracle's side): over all 65 536 gate patterns x 16
    up-values the device's bits equal the definition's wherever the exact product is further than the
    recipe's error (3.5 fp32 ulp) from a point where the 16-bit rounding flips; inside that band (counted
    below) they are one step of the 16-bit grid apart at most."""
    import oracle
    torch = gu.torch_mod()
    ups = synth.encode16(np.array([1.0, -0.37, 3.1, 1e-4, 250.0, 7e-3, 0.11, -33.0, 0.0, -0.0, 6e4, -2e-7,
                                   np.inf, 1.0009765625, -7.5, 2e-3]), dt)
    G = np.repeat(np.arange(65536, dtype=np.uint16), len(ups))
    U = np.tile(ups, 65536)
    want, margin = oracle.gated_input_plain(G, U, dt)
    Gd, Ud = gu.to_dev16(G), gu.to_dev16(U)
    out = torch.zeros_like(Gd)
    rs.rsparse_gated_input(Gd.data_ptr(), Ud.data_ptr(), out.data_ptr(), G.size, dt, gu.stream_ptr())
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint16)
    gd, wd = synth.decode16(got, dt), synth.decode16(want, dt)
    g_val, u_val = synth.decode16(G, dt), synth.decode16(U, dt)
    # Gates below -87: the recipe flushes silu to -0 there (|silu(g)| < 88 e^-87 = 1.5e-36), so the device
    # stores -0 * u where the definition still has a value of at most that size times |u| -- a documented
    # deviation of the recipe, checked as such; everywhere else NaN patterns must agree.
    low = g_val < -87.0
    fin_u = np.isfinite(u_val)
    assert np.all(gd[low & fin_u] == 0.0) and np.all(np.abs(wd[low & fin_u]) <= 1.5e-36 * np.abs(u_val[low & fin_u]))
    nan = np.isnan(wd)
    assert np.array_equal(np.isnan(gd[~low]), nan[~low])
    ok = ~nan & ~low
    band = oracle.RECIPE_BAND[dt]
    far = ok & (margin > band)
    assert np.array_equal(got[far], want[far])
    near = ok & ~far
    p_bits = 11 if dt == synth.F16 else 8
    step = 2.0 ** (1 - p_bits) * np.maximum(np.abs(gd[near]), np.abs(wd[near]))
    tiny = 2.0 ** (-24 if dt == synth.F16 else -133)
    assert np.array_equal(np.isfinite(wd[near]), np.isfinite(gd[near]))
    fin = np.isfinite(wd[near])
    assert np.all(np.abs(gd[near][fin] - wd[near][fin]) <= step[fin] + tiny)
    n_band = int(near.sum())
    n_diff = int((got[ok] != want[ok]).sum())
    print(f"dtype {dt}: {n_band} of {ok.sum()} cases within the band of {band:.2e} spacings; {n_diff} differ in bits")
    assert n_band < 0.01 * ok.sum()


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("B", [1, 3, 4, 8, 12, 32])
def test_gated_mlp_input(ragged, dt, B):
    """rsparse_linear_gated: x = round16(silu(g) * u) formed on the device (Sec. 3.1).  The oracle
    forms x by its own copy of the fp32 recipe; kept-channel lists must be equal, outputs within the
    usual bounds.  1-4 tokens: vector path (both launch forms); 8-32: matrix-core path and, with
    the row-major copy left out, the vector path in tiles of 8.  Values span fp16 subnormals to
    overflow, NaN and Inf included."""
    import oracle
    L = ragged[dt]
    pair = synth.GateUpPair(L.d_in, config=86, linear=B)
    g, u = pair.tokens(B)
    u *= np.exp(np.random.default_rng(B).uniform(-3, 3, size=u.shape))
    g[0, 1:3] = [40.0, -95.0]
    u[0, 4:6] = [1e-7, -3e4]
    if B > 1:                      # a NaN or Inf input turns every output of its token into NaN: keep token 0 finite at B = 1
        g[1, 0] = np.nan
        u[1, 3] = np.inf
    G16, U16 = synth.encode16(g, dt), synth.encode16(u, dt)
    X16 = oracle.gated_input(G16, U16, dt)
    tau = oracle.quantile_tau(oracle.gated_input(*[synth.encode16(a, dt) for a in pair.tokens(64, stream=synth.STREAM_CALIB)], dt), dt, 0.5)
    want = gu.oracle_linear(L, X16, tau)
    for rowmajor in (1, 0):
        layer = gu.prepare(L, tau, max_batch=B, out_dtype=rs.F32, dense_rowmajor=rowmajor)
        for launches in (1, 2):
            rs.rsparse_set_tuning(layer, launches=launches)
            Gd, Ud = gu.to_dev16(G16), gu.to_dev16(U16)
            Y = gu._alloc_out(layer, B)
            rs.rsparse_linear_gated(layer, Gd.data_ptr(), Ud.data_ptr(), B, Y.data_ptr(), gu.stream_ptr())
            got = {"Y": gu._read_out(layer, Y), "act": [rs.rsparse_last_active(layer, b) for b in range(B)],
                   "union": rs.rsparse_last_active(layer, -1)}
            gu.check_lists(got, want)
            gu.check_outputs(got["Y"], want["Y"], rs.F32)
        layer.destroy()


def test_gated_matches_ungated_on_the_materialised_input(ragged):
    """The gated entry equals rsparse_linear on x written out by the oracle's recipe: same lists, and
    outputs equal up to the order of the atomic adds."""
    import oracle
    L = ragged[synth.BF16]
    g, u = synth.GateUpPair(L.d_in, config=86, linear=99).tokens(2)
    G16, U16 = synth.encode16(g, L.dtype), synth.encode16(u, L.dtype)
    X16 = oracle.gated_input(G16, U16, L.dtype)
    tau = oracle.quantile_tau(X16, L.dtype, 0.5)
    layer = gu.prepare(L, tau, max_batch=2, out_dtype=rs.F32)
    plain = gu.run_linear(layer, X16)
    Gd, Ud = gu.to_dev16(G16), gu.to_dev16(U16)
    Y = gu._alloc_out(layer, 2)
    rs.rsparse_linear_gated(layer, Gd.data_ptr(), Ud.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    fused = gu._read_out(layer, Y)
    for b in range(2):
        assert np.array_equal(rs.rsparse_last_active(layer, b), plain["act"][b])
    assert np.linalg.norm(fused - plain["Y"]) <= 1e-5 * np.linalg.norm(plain["Y"])
    with pytest.raises(rs.RSparseError):
        rs.rsparse_linear_gated(layer, 0, Ud.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    layer.destroy()


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("B", [1, 3, 8, 12])
def test_mlp_gate_up_with_fused_activation(dt, B):
    """rsparse_mlp_gate_up: H = round(silu(round g) * round u) (Sec. 3.1) from the two R-Sparse
    projections.  One launch on the vector path (1-8 tokens without the row-major copy), the
    two-layers-then-elementwise fallback elsewhere; kept-channel lists of both layers must equal the
    oracle's, H within the 16-bit output bounds.  Different rank and threshold per layer."""
    import oracle
    torch = gu.torch_mod()
    Lg = synth.make_layer(1032, 1096, 40, dt, config=87, linear=0)
    Lu = synth.make_layer(1032, 1096, 24, dt, config=87, linear=1)
    X16, src = gu.tokens_for(Lg, B, linear=60 + B)
    tg, tu = gu.calibrated_tau(Lg, src, 0.5), gu.calibrated_tau(Lg, src, 0.6)
    wg, wu = gu.oracle_linear(Lg, X16, tg), gu.oracle_linear(Lu, X16, tu)
    h_want = synth.decode16(oracle.gated_input(synth.encode16(wg["Y"], dt), synth.encode16(wu["Y"], dt), dt), dt)
    for rowmajor, launches in ((0, 1), (0, 2), (1, 1)):
        gate = gu.prepare(Lg, tg, max_batch=B, dense_rowmajor=rowmajor)
        up = gu.prepare(Lu, tu, max_batch=B, dense_rowmajor=rowmajor)
        rs.rsparse_set_tuning(gate, launches=launches)
        Xd = gu.to_dev16(X16)
        H = gu._alloc_out(gate, B)
        for rep in range(2):                                  # twice: the shared counters must be back at zero
            H.fill_(0x7FFF)
            rs.rsparse_mlp_gate_up(gate, up, Xd.data_ptr(), B, H.data_ptr(), gu.stream_ptr())
            rs.rsparse_synchronize(gate)
            rs.rsparse_synchronize(up)
            gu.check_outputs(gu._read_out(gate, H), h_want, gate.cfg.out_dtype)
            for layer, w in ((gate, wg), (up, wu)):
                got = {"act": [rs.rsparse_last_active(layer, b) for b in range(B)], "union": rs.rsparse_last_active(layer, -1)}
                gu.check_lists(got, w)
        # the handles still work on their own afterwards
        one = gu.run_linear(up, X16)
        gu.check_outputs(one["Y"], wu["Y"], up.cfg.out_dtype)
        with pytest.raises(rs.RSparseError):
            rs.rsparse_mlp_gate_up(gate, gate, Xd.data_ptr(), B, H.data_ptr(), gu.stream_ptr())
        gate.destroy()
        up.destroy()


def test_bounded_wait_runs_out_and_the_handle_recovers(ragged):
    """Error path of the one-launch kernel, forced from the host: stage 1 publishes nothing and the
    wait bound is a few polls, so every kernel still ends normally; the call is reported invalid by
    rsparse_synchronize and by rsparse_last_active, and the next call on the handle is correct again."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 2, linear=77)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=2, out_dtype=rs.F32)
    with pytest.raises(rs.RSparseError):
        rs.rsparse_set_tuning(layer, launches=1, debug_skip_stage1=1)              # needs a short bound
    rs.rsparse_set_tuning(layer, launches=1, debug_skip_stage1=1, debug_wait_polls=4)
    Xd = gu.to_dev16(X16)
    Y = gu._alloc_out(layer, 2)
    rs.rsparse_linear(layer, Xd.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    with pytest.raises(rs.RSparseError) as e:
        rs.rsparse_synchronize(layer)
    assert e.value.status == rs.binding.EHIP
    rs.rsparse_set_tuning(layer, launches=1)
    for _ in range(2):
        got = gu.run_linear(layer, X16)
        rs.rsparse_synchronize(layer)
        want = gu.oracle_linear(L, X16, tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_dense_ref_both_kernels(ragged, dt):
    import oracle
    L = ragged[dt]
    X16, _ = gu.tokens_for(L, 5)
    want = oracle.dense_linear(L.W16, X16, L.dtype, L.dtype, nthreads=8)
    for out in (None, rs.F32):
        layer = gu.prepare(L, 0.5, max_batch=8, out_dtype=out, dense_rowmajor=1)
        for kernel, min_b in ((1, 33), (2, 33), (0, 33), (0, 0)):     # vector kernels, then default (MFMA from 2 tokens)
            rs.rsparse_set_tuning(layer, dense_kernel=kernel, mfma_min_batch=min_b)
            for B in (1, 5):
                got = gu.run_dense(layer, X16[:B])
                gu.check_outputs(got, want[:B], layer.cfg.out_dtype)
        layer.destroy()


def test_determinism_of_lists_and_bounded_output_jitter(config0):
    L = config0
    src = synth.DModelInput(L.d_in, config=0, linear=0)
    tau = gu.calibrated_tau(L, src, 0.5)
    X16 = synth.encode16(src.tokens(1, offset=3), L.dtype)
    layer = gu.prepare(L, tau, out_dtype=rs.F32)
    first = gu.run_linear(layer, X16)
    for _ in range(20):
        again = gu.run_linear(layer, X16)
        assert np.array_equal(again["act"][0], first["act"][0])
        # fp32 atomics: summation order may differ between runs, within accumulation rounding
        assert np.linalg.norm(again["Y"] - first["Y"]) <= 1e-5 * np.linalg.norm(first["Y"])


@pytest.mark.parametrize("shape", [(4096, 11008, 512, "dmodel"), (11008, 4096, 512, "down")])
def test_config1_shapes_sparsity_sweep(shape):
    """configs[1]: Llama-2-7B MLP shapes, bf16, r = 512, tau at 40 / 50 / 70 % sparsity."""
    d_in, d_out, r, kind = shape
    L = synth.make_layer(d_in, d_out, r, synth.BF16, config=1, linear=0 if kind == "dmodel" else 2)
    X16, src = gu.tokens_for(L, 2, kind=kind, config=1, linear=0 if kind == "dmodel" else 2)
    for s in (0.4, 0.5, 0.7):
        tau = gu.calibrated_tau(L, src, s)
        got, _ = _parity(L, X16[0], tau)
        assert abs(len(got["act"][0]) / d_in - (1 - s)) < 0.05
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16[1], tau, out_dtype=rs.F32)


def test_config1_as_benchmarked_grouped_and_replayed():
    """The launch configuration bench.py times: gate and up (4096 -> 11008) in one grouped call, then
    down (11008 -> 4096), bf16, r = 512, 50 % sparsity, default launch shapes, captured into a HIP
    graph and replayed; every output of every replay against the oracle, both launch forms."""
    import oracle
    torch = gu.torch_mod()
    dt = synth.BF16
    specs = [(4096, 11008, "dmodel", 0), (4096, 11008, "dmodel", 1), (11008, 4096, "down", 2)]
    Ls = [synth.random_layer(d_in, d_out, 512, dt, seed=1100 + lin) for d_in, d_out, _, lin in specs]
    src_m = synth.DModelInput(4096, config=1, linear=0)
    src_d = synth.DownInput(11008, config=1, linear=2)
    taus = [gu.calibrated_tau(Ls[0], src_m, 0.5), gu.calibrated_tau(Ls[1], src_m, 0.5), gu.calibrated_tau(Ls[2], src_d, 0.5)]
    xm = synth.encode16(src_m.tokens(1, offset=3), dt)
    xd = synth.encode16(src_d.tokens(1, offset=3), dt)
    want = [oracle.rsparse_linear(L.W16, L.U16, L.SV16, x, dt, dt, tau, nthreads=8)
            for L, x, tau in zip(Ls, (xm, xm, xd), taus)]
    layers = [gu.prepare(L, tau, max_batch=1, dense_rowmajor=1) for L, tau in zip(Ls, taus)]
    xm_d, xd_d = gu.to_dev16(xm), gu.to_dev16(xd)
    Ys = [gu._alloc_out(layer, 1) for layer in layers]

    def step(sptr):
        rs.rsparse_linear_group(layers[:2], xm_d.data_ptr(), 1, [Ys[0].data_ptr(), Ys[1].data_ptr()], sptr)
        rs.rsparse_linear(layers[2], xd_d.data_ptr(), 1, Ys[2].data_ptr(), sptr)

    for launches in (1, 2):
        for layer in layers:
            rs.rsparse_set_tuning(layer, launches=launches)
        step(gu.stream_ptr())
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            for Y in Ys:
                Y.fill_(0x7FFF)
            graph.replay()
            torch.cuda.synchronize()
            for layer, Y, w in zip(layers, Ys, want):
                rs.rsparse_synchronize(layer)
                gu.check_outputs(gu._read_out(layer, Y), w["Y"], layer.cfg.out_dtype)
                assert np.array_equal(rs.rsparse_last_active(layer, 0), w["act"][0])
    for layer in layers:
        layer.destroy()


def test_largest_shape_sampled():
    """Llama-3-70B gate/up shape (8192 -> 28672, r = 1024), cheap random operands; the oracle checks
    every output of one token (about a second of CPU)."""
    L = synth.random_layer(8192, 28672, 1024, synth.BF16, seed=4001)
    X16, src = gu.tokens_for(L, 1, config=4)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16, tau)
    L2 = synth.random_layer(28672, 8192, 1024, synth.BF16, seed=4002)
    X16, src = gu.tokens_for(L2, 2, kind="down", config=4)
    tau = gu.calibrated_tau(L2, src, 0.5)
    _parity(L2, X16, tau, out_dtype=rs.F32)


@pytest.mark.parametrize("B", [1, 3, 8])
def test_group_of_layers_sharing_one_input(B):
    """q/k/v- or gate/up-style groups: one pair of launches, results equal separate calls and the oracle.
    Different d_out, rank and tau per layer."""
    import oracle
    specs = [(1032, 1096, 40, 0.5), (1032, 520, 0, 0.4), (1032, 2056, 64, 0.6)]
    Ls = [synth.make_layer(d_in, d_out, r, synth.BF16, config=84, linear=i) for i, (d_in, d_out, r, _) in enumerate(specs)]
    X16, src = gu.tokens_for(Ls[0], B, linear=B)
    taus = [gu.calibrated_tau(Ls[0], src, s) for (_, _, _, s) in specs]
    for out in (None, rs.F32):
        layers = [gu.prepare(L, tau, max_batch=B, out_dtype=out, dense_rowmajor=1) for L, tau in zip(Ls, taus)]
        if out is None:      # mixed launch-shape overrides inside one group: the first layer's block size rules
            rs.rsparse_set_tuning(layers[0], waves=4, splits=5)
            rs.rsparse_set_tuning(layers[2], waves=8, splits=3, lowrank_rows=32)
        Xd = gu.to_dev16(X16)
        Ys = [gu._alloc_out(layer, B) for layer in layers]
        rs.rsparse_linear_group(layers, Xd.data_ptr(), B, [y.data_ptr() for y in Ys], gu.stream_ptr())
        for L, tau, layer, Y in zip(Ls, taus, layers, Ys):
            got = {"Y": gu._read_out(layer, Y), "act": [rs.rsparse_last_active(layer, b) for b in range(B)],
                   "union": rs.rsparse_last_active(layer, -1)}
            want = gu.oracle_linear(L, X16, tau)
            gu.check_lists(got, want)
            gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
        for kernel in (1, 2):
            rs.rsparse_set_tuning(layers[0], dense_kernel=kernel)
            Ys = [gu._alloc_out(layer, B) for layer in layers]
            rs.rsparse_dense_ref_group(layers, Xd.data_ptr(), B, [y.data_ptr() for y in Ys], gu.stream_ptr())
            for L, layer, Y in zip(Ls, layers, Ys):
                want = oracle.dense_linear(L.W16, X16, L.dtype, L.dtype, nthreads=8)
                gu.check_outputs(gu._read_out(layer, Y), want, layer.cfg.out_dtype)
        for layer in layers:
            layer.destroy()


def test_group_argument_errors(ragged):
    L = ragged[synth.F16]
    other = synth.make_layer(520, 264, 0, synth.F16, config=82, linear=0)
    a, b = gu.prepare(L, 0.5), gu.prepare(other, 0.5)
    X16, _ = gu.tokens_for(L, 1)
    Xd = gu.to_dev16(X16)
    Y = gu._alloc_out(a, 1)
    with pytest.raises(rs.RSparseError):       # different d_in
        rs.rsparse_linear_group([a, b], Xd.data_ptr(), 1, [Y.data_ptr(), Y.data_ptr()], gu.stream_ptr())
    with pytest.raises(rs.RSparseError):       # same handle twice
        rs.rsparse_linear_group([a, a], Xd.data_ptr(), 1, [Y.data_ptr(), Y.data_ptr()], gu.stream_ptr())
    with pytest.raises(rs.RSparseError):       # batch above max_batch
        rs.rsparse_linear(a, Xd.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    with pytest.raises(rs.RSparseError):       # misaligned X
        rs.rsparse_linear(a, Xd.data_ptr() + 2, 1, Y.data_ptr(), gu.stream_ptr())


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("B", [5, 8, 9, 16, 17, 32])
@pytest.mark.parametrize("mask_mode", [0, 1])
def test_matrix_core_path_batches(ragged, dt, B, mask_mode):
    """5..32 tokens with the row-major copy of W present: the MFMA path (dense masked GEMM, stage 1 and
    stage 2 on matrix cores).  Same oracle, same tolerances; ragged K chunk (1032 = 32*32 + 8) and rows."""
    L = ragged[dt]
    X16, src = gu.tokens_for(L, B, linear=40 + B)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16, tau, out_dtype=rs.F32, batch_mask_mode=mask_mode, dense_rowmajor=1)
    _parity(L, X16, tau, batch_mask_mode=mask_mode, dense_rowmajor=1)


def test_matrix_core_path_matches_vector_path_and_edges(ragged):
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 20, linear=77)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=32, out_dtype=rs.F32, dense_rowmajor=1)
    a = gu.run_linear(layer, X16)
    rs.rsparse_set_tuning(layer, mfma_min_batch=33)
    b = gu.run_linear(layer, X16)
    gu.check_lists(a, b)
    assert np.linalg.norm(a["Y"] - b["Y"]) <= 3e-5 * np.linalg.norm(b["Y"])
    rs.rsparse_set_tuning(layer, mfma_min_batch=0)
    # same handle, smaller batches in between (vector path), then back: scratch stays consistent
    for B in (3, 20, 1, 12):
        got = gu.run_linear(layer, X16[:B])
        want = gu.oracle_linear(L, X16[:B], tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    # thresholds at the extremes and a NaN token
    for t2 in (-INF, INF):
        rs.rsparse_set_tau(layer, t2)
        got = gu.run_linear(layer, X16[:16])
        want = gu.oracle_linear(L, X16[:16], t2)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    rs.rsparse_set_tau(layer, tau)
    Xn = X16[:16].copy()
    Xn[5, 9] = 0x7FC0
    got = gu.run_linear(layer, Xn)
    want = gu.oracle_linear(L, Xn, tau)
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], rs.F32)
    assert np.all(np.isnan(got["Y"][5])) and np.all(np.isfinite(got["Y"][4]))
    layer.destroy()


@pytest.mark.parametrize("shape", [(4096, 1024, 128, 16), (4096, 4096, 512, 16), (8192, 8192, 1024, 32)])
def test_matrix_core_path_llama3_shapes(shape):
    """configs[3]/[4] shapes (GQA k/v 4096->1024, q/o 4096->4096, 70B q/o 8192->8192) at 16 / 32 tokens."""
    d_in, d_out, r, B = shape
    L = synth.random_layer(d_in, d_out, r, synth.BF16, seed=3000 + d_out)
    X16, src = gu.tokens_for(L, B, config=3, linear=B)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16, tau, dense_rowmajor=1)
    _parity(L, X16, tau, out_dtype=rs.F32, dense_rowmajor=1)


@pytest.mark.parametrize("B", [1, 8])
def test_hip_graph_replays_match_eager_and_oracle(ragged, B):
    """The hot calls are capturable: a captured graph of one call is replayed several times, with new
    token values written into the same input buffer and eager work in between; every replay must equal
    the eager call on the same input and the oracle (scratch is re-zeroed by the kernels themselves)."""
    torch = gu.torch_mod()
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 4 * B, linear=60 + B)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=B, out_dtype=rs.F32, dense_rowmajor=1)
    Xd = gu.to_dev16(X16[:B])
    Y = gu._alloc_out(layer, B)
    Ye = gu._alloc_out(layer, B)
    rs.rsparse_linear(layer, Xd.data_ptr(), B, Y.data_ptr(), gu.stream_ptr())      # load everything first
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rs.rsparse_linear(layer, Xd.data_ptr(), B, Y.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        xb = X16[rep * B:(rep + 1) * B]
        Xd.copy_(torch.from_numpy(np.ascontiguousarray(xb).view(np.int16)))
        Y.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = Y.cpu().numpy().astype(np.float64)
        rs.rsparse_linear(layer, Xd.data_ptr(), B, Ye.data_ptr(), gu.stream_ptr())  # eager, between replays
        torch.cuda.synchronize()
        eager = Ye.cpu().numpy().astype(np.float64)
        want = gu.oracle_linear(L, xb, tau)
        gu.check_outputs(got, want["Y"], rs.F32)
        assert np.linalg.norm(got - eager) <= 1e-5 * np.linalg.norm(eager)
        assert np.array_equal(rs.rsparse_last_active(layer, 0), want["act"][0])
    layer.destroy()


@pytest.mark.parametrize("seed", list(range(6)))
def test_random_shapes_and_settings(seed):
    """Seeded sweep over small random layers: every dimension a multiple of 8 from 8 up, ranks from 0 to
    full, 1-32 tokens, both dtypes, both compare modes, both mask modes, with and without the row-major
    copy, both launch forms, random launch shapes.  Lists equal, outputs within the fp32-output bound."""
    rng = np.random.default_rng(1234 + seed)
    for case in range(8):
        d_in = 8 * int(rng.integers(1, 150))
        d_out = 8 * int(rng.integers(1, 200))
        rank = 8 * int(rng.integers(0, min(d_in, d_out) // 8 + 1))
        if rng.random() < 0.5:
            rank = min(rank, 8 * int(rng.integers(0, 9)))
        dt = int(rng.integers(0, 2))
        B = int(rng.choice([1, 1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 32]))
        cmp_mode, mask_mode, rowmajor = int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2))
        L = synth.random_layer(d_in, d_out, rank, dt, seed=9000 + 100 * seed + case)
        src = synth.DModelInput(d_in, config=88, linear=10 * seed + case)
        X16 = synth.encode16(src.tokens(B), dt)
        s_level = float(rng.choice([0.0, 0.3, 0.5, 0.5, 0.8, 1.0]))
        tau = gu.calibrated_tau(L, src, s_level) if 0.0 < s_level < 1.0 else (-INF if s_level == 0.0 else INF)
        tuning = {"launches": int(rng.integers(1, 3))}
        if rng.random() < 0.5:
            tuning.update(splits=int(rng.integers(1, 40)), waves=int(rng.choice([1, 2, 4, 8])))
        if rng.random() < 0.3:
            tuning.update(lowrank_rows=int(rng.integers(1, 33)))
        label = dict(d_in=d_in, d_out=d_out, rank=rank, dt=dt, B=B, cmp=cmp_mode, mask=mask_mode, rowmajor=rowmajor,
                     s=s_level, **tuning)
        print("case", label, flush=True)
        _parity(L, X16, tau, out_dtype=rs.F32, tuning=tuning, cmp_mode=cmp_mode, batch_mask_mode=mask_mode,
                dense_rowmajor=rowmajor)


def test_prepare_with_the_host_svd_end_to_end():
    """rsparse_prepare (the first call of the path: host SVD -> stored 16-bit factors -> pack -> upload) followed by
    rsparse_get_factors / rsparse_get_config: the oracle consumes exactly the factor bits the library stored, and
    the layer must match it; the factors themselves are checked against the generator's closed form through the
    product they stand for (Eckart-Young: the best rank-r approximation), not vector by vector."""
    for d_in, d_out, r, dt in ((520, 264, 24, synth.BF16), (264, 520, 16, synth.F16)):
        L = synth.make_layer(d_in, d_out, r, dt, config=89, linear=dt)
        src = synth.DModelInput(d_in, config=89, linear=dt)
        tau = gu.calibrated_tau(L, src, 0.5)
        cfg = rs.make_config(d_in, d_out, r, tau, dt, max_batch=2, out_dtype=rs.F32, cmp_mode=1)
        layer = rs.rsparse_prepare(cfg, L.W16)
        back = rs.rsparse_get_config(layer)
        for f in ("d_in", "d_out", "rank", "max_batch", "dtype", "out_dtype", "cmp_mode", "batch_mask_mode", "dense_rowmajor", "strip_cols"):
            assert getattr(back, f) == getattr(cfg, f), f
        assert back.tau == np.float32(tau)
        U16, SV16 = rs.rsparse_get_factors(layer)
        assert U16.shape == (d_out, r) and SV16.shape == (r, d_in)
        # the stored factors reproduce the top-r part of W: || U (S V^T) - U_r diag(s_r) V_r^T ||_F is at the level of
        # 16-bit rounding of the factors
        prod = synth.decode16(U16, dt) @ synth.decode16(SV16, dt)
        best = (L.U[:, :r] * L.sigma[:r]) @ L.V[:, :r].T
        assert np.linalg.norm(prod - best) <= (2e-2 if dt == synth.BF16 else 4e-3) * np.linalg.norm(best)
        X16 = synth.encode16(src.tokens(2), dt)
        got = gu.run_linear(layer, X16)
        import oracle
        want = oracle.rsparse_linear(L.W16, U16, SV16, X16, dt, dt, tau, cmp_mode=1, nthreads=8)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
        rs.rsparse_set_tau(layer, 2.0 * tau)
        assert rs.rsparse_get_config(layer).tau == np.float32(2.0 * tau)
        # the byte model of the handle equals the shape-only model
        assert rs.rsparse_required_bytes(layer, 2, 100) == rs.rsparse_io_model(cfg, 2, 100)[0]
        assert rs.rsparse_dense_bytes(layer, 2) == rs.rsparse_io_model(cfg, 2, 0)[1]
        layer.destroy()


def test_prepare_with_the_host_svd_on_a_4096_layer(config0):
    """The same on configs[0]'s 4096 x 4096 layer (power-law spectrum; r = 64 keeps the host SVD to seconds)."""
    import oracle
    dt = synth.F16
    L = config0
    src = synth.DModelInput(4096, config=89, linear=3)
    tau = gu.calibrated_tau(L, src, 0.5)
    cfg = rs.make_config(4096, 4096, 64, tau, dt)
    layer = rs.rsparse_prepare(cfg, L.W16)
    U16, SV16 = rs.rsparse_get_factors(layer)
    # the top 64 components of the generator's closed form, up to fp16 rounding of W and of the factors
    best = (L.U[:, :64] * L.sigma[:64]) @ L.V[:, :64].T
    assert np.linalg.norm(synth.decode16(U16, dt) @ synth.decode16(SV16, dt) - best) <= 2e-2 * np.linalg.norm(best)
    X16 = synth.encode16(src.tokens(1), dt)
    got = gu.run_linear(layer, X16)
    want = oracle.rsparse_linear(L.W16, U16, SV16, X16, dt, dt, tau, nthreads=8)
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], dt)
    layer.destroy()


def test_nothing_is_written_past_the_end_of_the_outputs(ragged):
    """Canaries around Y: the output buffer sits inside a larger allocation filled with a pattern; after calls
    through every path (one and two launches, 8-token tiles, matrix cores, strips, dense baselines) only the
    batch x d_out outputs may have changed."""
    torch = gu.torch_mod()
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 9, linear=12)
    tau = gu.calibrated_tau(L, src, 0.5)
    pad = 4096                                                   # 16-bit words of canary on each side
    for kw, tuning, B in ((dict(), dict(), 1), (dict(), dict(launches=2), 3), (dict(), dict(), 8),
                          (dict(dense_rowmajor=1), dict(), 9), (dict(strip_cols=32), dict(), 1),
                          (dict(strip_cols=64), dict(splits=3), 9), (dict(out_dtype=rs.F32), dict(), 2)):
        layer = gu.prepare(L, tau, max_batch=B, **kw)
        rs.rsparse_set_tuning(layer, **tuning)
        words = (2 if layer.cfg.out_dtype == rs.F32 else 1) * B * L.d_out
        buf = torch.full((pad + words + pad,), 0x5A5A, dtype=torch.int16, device="cuda")
        Y = buf[pad:pad + words]
        assert Y.data_ptr() % 16 == 0
        Xd = gu.to_dev16(X16[:B])
        for fn in (rs.rsparse_linear, rs.rsparse_dense_ref, rs.rsparse_linear_static if B <= 8 else rs.rsparse_linear):
            buf.fill_(0x5A5A)
            fn(layer, Xd.data_ptr(), B, Y.data_ptr(), gu.stream_ptr())
            torch.cuda.synchronize()
            host = buf.cpu().numpy()
            assert np.all(host[:pad] == 0x5A5A) and np.all(host[pad + words:] == 0x5A5A), (kw, tuning, B, fn.__name__)
            assert np.any(host[pad:pad + words] != 0x5A5A)
        layer.destroy()
