"""GPU parity of the strip layout (rsparse_config.strip_cols > 0): the same layer, run by the strip kernel -- one
workgroup (or a few channel splits) per strip of output columns, every wave on a fixed range of input channels,
stage 1 of the low-rank part handed over inside the launch through generation-tagged entries.  Everything is
compared with the fp64 CPU oracle through the C ABI: kept-channel lists equal, outputs within the stated
tolerances."""
import numpy as np
import pytest

import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
INF = float("inf")


@pytest.fixture(scope="module")
def ragged():
    """Ragged in every direction: 1096 columns = 34 strips of 32 + 8, 1032 channels = 129 groups of 8."""
    return {dt: synth.make_layer(1032, 1096, 40, dt, config=81, linear=dt) for dt in (synth.F16, synth.BF16)}


def _parity(L, X16, tau, strip_cols, out_dtype=None, max_batch=None, tuning=None, **cfg_kw):
    X16 = np.atleast_2d(X16)
    layer = gu.prepare(L, tau, max_batch=max_batch or X16.shape[0], out_dtype=out_dtype, strip_cols=strip_cols, **cfg_kw)
    assert rs.rsparse_get_config(layer).strip_cols == strip_cols
    if tuning:
        rs.rsparse_set_tuning(layer, **tuning)
    got = gu.run_linear(layer, X16)
    rs.rsparse_synchronize(layer)
    want = gu.oracle_linear(L, X16, tau, cmp_mode=cfg_kw.get("cmp_mode", 0),
                            batch_mask_mode=cfg_kw.get("batch_mask_mode", 0))
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
    layer.destroy()
    return got, want


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("W", [32, 64, 128, 256, 512])
@pytest.mark.parametrize("out", [None, rs.F32])
def test_every_strip_width(ragged, dt, W, out):
    L = ragged[dt]
    X16, src = gu.tokens_for(L, 2, linear=dt)
    tau = gu.calibrated_tau(L, src, 0.5)
    for b in range(2):
        got, _ = _parity(L, X16[b], tau, W, out_dtype=out)
        assert 0.3 * L.d_in < len(got["act"][0]) < 0.7 * L.d_in


@pytest.mark.parametrize("W", [32, 128])
@pytest.mark.parametrize("splits", [1, 2, 3, 7, 40])
def test_channel_splits(ragged, W, splits):
    """One workgroup per strip (no sums cross workgroups) up to many channel splits per strip (partial sums meet in
    atomics, the last workgroup of a strip stores); 40 splits x 8 waves leaves ranges of less than one group of 8."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 4, linear=3)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16[0], tau, W, out_dtype=rs.F32, tuning=dict(splits=splits))
    _parity(L, X16, tau, W, out_dtype=rs.F32, tuning=dict(splits=splits))


def test_edge_thresholds_and_ties(ragged):
    L = ragged[synth.F16]
    X16, _ = gu.tokens_for(L, 1)
    for tau in (-INF, 0.0, INF, 1e30, 3.0e-45, -1.0):
        for mode in (0, 1):
            _parity(L, X16, tau, 64, out_dtype=rs.F32, cmp_mode=mode)
    Lb = ragged[synth.BF16]
    x = np.where(np.arange(Lb.d_in) % 3 == 0, -0.75, 0.75)
    Xt = synth.encode16(x, Lb.dtype)
    got0, _ = _parity(Lb, Xt, 0.75, 32, cmp_mode=0)
    got1, _ = _parity(Lb, Xt, 0.75, 32, cmp_mode=1)
    assert len(got0["act"][0]) == Lb.d_in and len(got1["act"][0]) == 0
    # the strict compare is implemented as >= the next fp32: thresholds next to a tie, and the largest finite one
    for tau in (np.nextafter(np.float32(0.75), np.float32(0)), np.nextafter(np.float32(0.75), np.float32(1)),
                np.float32(3.4028235e38)):
        for mode in (0, 1):
            _parity(Lb, Xt, float(tau), 32, cmp_mode=mode)


def test_nan_inf_and_negative_zero_inputs(ragged):
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 1)
    tau = gu.calibrated_tau(L, src, 0.5)
    X = X16[0].copy()
    X[5], X[77], X[8] = 0x7C00, 0xFC00, 0x8000          # +inf and -inf are kept, -0 is not
    got, _ = _parity(L, X, tau, 64, out_dtype=rs.F32)
    assert 5 in got["act"][0] and 77 in got["act"][0] and 8 not in got["act"][0]
    X[9] = 0x7E00                                       # NaN: never kept, poisons every output through the low-rank part
    got, _ = _parity(L, X, tau, 64, out_dtype=rs.F32)
    assert 9 not in got["act"][0] and np.all(np.isnan(got["Y"]))


def test_rank_zero_and_subnormal_weights():
    L0 = synth.make_layer(520, 264, 0, synth.F16, config=82, linear=0)
    X16, src = gu.tokens_for(L0, 2)
    tau = gu.calibrated_tau(L0, src, 0.6)
    _parity(L0, X16[0], tau, 32, out_dtype=rs.F32)
    _parity(L0, X16, tau, 128, out_dtype=rs.F32, tuning=dict(splits=2))
    L = synth.make_layer(264, 520, 8, synth.F16, config=83, linear=0)
    W = synth.decode16(L.W16, L.dtype)
    L.W16 = synth.encode16(W * (3e-5 / np.max(np.abs(W))), L.dtype)            # every weight an fp16 subnormal
    L.rank, L.U16, L.SV16 = 0, L.U16[:, :0], L.SV16[:0]
    Xs, _ = gu.tokens_for(L, 1)
    _, want = _parity(L, Xs, 0.5, 64, out_dtype=rs.F32)
    assert np.linalg.norm(want["Y"]) > 0


@pytest.mark.parametrize("B", [2, 3, 4, 5, 8, 9, 16, 32])
@pytest.mark.parametrize("mask_mode", [0, 1])
def test_batches(ragged, B, mask_mode):
    """2 .. 32 tokens on the vector path (batch tiles of up to 8 tokens; per-token masks or the union mask)."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, B, linear=B)
    tau = gu.calibrated_tau(L, src, 0.5)
    _parity(L, X16, tau, 64, out_dtype=rs.F32, batch_mask_mode=mask_mode)
    _parity(L, X16, tau, 32, batch_mask_mode=mask_mode, tuning=dict(splits=1))


@pytest.mark.parametrize("launches", [1, 2])
@pytest.mark.parametrize("B", [1, 3, 8, 12])
def test_reused_handle_both_launch_forms(ragged, launches, B):
    """Back-to-back calls on one handle with different kept sets: the generation hand-off needs no reset between
    calls, the split strips' accumulators and counters are back at zero after every call.  launches = 2: stage 1 in
    a launch of its own, then the strip kernel."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, B, linear=40 + B)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=B, out_dtype=rs.F32, strip_cols=64)
    rs.rsparse_set_tuning(layer, launches=launches)
    for t in (tau, -INF, gu.calibrated_tau(L, src, 0.7), INF, tau):
        rs.rsparse_set_tau(layer, t)
        got = gu.run_linear(layer, X16)
        rs.rsparse_synchronize(layer)
        want = gu.oracle_linear(L, X16, t)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


def test_smaller_batches_on_a_large_handle(ragged):
    """max_batch = 32 but calls of 1 .. 32 tokens: the token slots a call does not use still get the call's
    generation, and rows of t left by larger calls are never mistaken for the current ones."""
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 32)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=32, out_dtype=rs.F32, strip_cols=32)
    for B in (32, 1, 9, 2, 32, 5):
        Xb = X16[32 - B:]                       # different tokens in the same slots
        got = gu.run_linear(layer, Xb)
        rs.rsparse_synchronize(layer)
        want = gu.oracle_linear(L, Xb, tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


def test_long_ranges_need_several_list_segments():
    """d_in = 16384 with one workgroup per strip: 2048 channels per wave.  With every channel kept a wave's list
    does not fit its LDS in one piece, so it is built and streamed in segments."""
    L = synth.random_layer(16384, 72, 24, synth.BF16, seed=91)
    src = synth.DModelInput(L.d_in, config=91, linear=0)
    X16 = synth.encode16(src.tokens(2), L.dtype)
    tau = gu.calibrated_tau(L, src, 0.5)
    for t in (-INF, tau, INF):
        _parity(L, X16[0], t, 32, out_dtype=rs.F32, tuning=dict(splits=1))
    _parity(L, X16, -INF, 64, out_dtype=rs.F32, tuning=dict(splits=1))


def test_one_workgroup_per_strip_is_bit_reproducible(ragged):
    """No sums cross workgroups and every wave adds its rows in a fixed order: 20 calls give identical bits."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 1, linear=5)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, out_dtype=rs.F32, strip_cols=32)
    rs.rsparse_set_tuning(layer, splits=1)
    torch = gu.torch_mod()
    Xd = gu.to_dev16(X16)
    outs = []
    for _ in range(20):
        Y = gu._alloc_out(layer, 1)
        rs.rsparse_linear(layer, Xd.data_ptr(), 1, Y.data_ptr(), gu.stream_ptr())
        torch.cuda.synchronize()
        outs.append(Y.cpu().numpy().view(np.uint32).copy())
    assert all(np.array_equal(o, outs[0]) for o in outs)
    layer.destroy()


def test_bounded_wait_runs_out_and_the_handle_recovers(ragged):
    """The error path, forced from the host: stage 1 publishes nothing and the bound on re-reads is a few polls, so
    every workgroup still ends normally; the call is reported invalid and the next one is correct again."""
    L = ragged[synth.BF16]
    X16, src = gu.tokens_for(L, 2, linear=77)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=2, out_dtype=rs.F32, strip_cols=64)
    rs.rsparse_set_tuning(layer, debug_skip_stage1=1, debug_wait_polls=4)
    Xd = gu.to_dev16(X16)
    Y = gu._alloc_out(layer, 2)
    rs.rsparse_linear(layer, Xd.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    with pytest.raises(rs.RSparseError) as e:
        rs.rsparse_synchronize(layer)
    assert e.value.status == rs.binding.EHIP
    rs.rsparse_set_tuning(layer)
    for _ in range(2):
        got = gu.run_linear(layer, X16)
        rs.rsparse_synchronize(layer)
        want = gu.oracle_linear(L, X16, tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


@pytest.mark.parametrize("splits", [1, 3])
def test_graph_replay(ragged, splits):
    """The call captured into a HIP graph and replayed: every replay runs with the arguments of the capture, so the
    generation of the hand-off must come from device memory.  Replays are interleaved with eager calls on other
    tokens and synchronisations, and each is checked against the oracle."""
    torch = gu.torch_mod()
    L = ragged[synth.F16]
    X16, src = gu.tokens_for(L, 6, linear=9)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=2, out_dtype=rs.F32, strip_cols=64)
    rs.rsparse_set_tuning(layer, splits=splits)
    Xd = gu.to_dev16(X16[:2].copy())
    Y = gu._alloc_out(layer, 2)
    rs.rsparse_linear(layer, Xd.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rs.rsparse_linear(layer, Xd.data_ptr(), 2, Y.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for rep in range(5):
        Xr = X16[(rep % 3) * 2:(rep % 3) * 2 + 2]
        Xd.copy_(gu.to_dev16(Xr))                        # new tokens in the captured buffer
        Y.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        want = gu.oracle_linear(L, Xr, tau)
        gu.check_outputs(Y.cpu().numpy().astype(np.float64), want["Y"], rs.F32)
        # an eager call on the same handle in between (other tokens), then its own check
        Xe = X16[4:6] if rep % 2 else X16[2:4]
        got = gu.run_linear(layer, Xe)
        rs.rsparse_synchronize(layer)
        we = gu.oracle_linear(L, Xe, tau)
        gu.check_lists(got, we)
        gu.check_outputs(got["Y"], we["Y"], rs.F32)
    layer.destroy()


def test_grouped_layers_and_mixed_layouts():
    """q / k / v: three strip layers of one width share a launch; a group whose layers differ in layout falls back
    to one call per layer.  Results equal the oracle's for each layer."""
    torch = gu.torch_mod()
    dt = synth.BF16
    shapes = [(520, 264, 16), (520, 1096, 40), (520, 72, 8)]
    Ls = [synth.make_layer(d_in, d_out, r, dt, config=84, linear=i) for i, (d_in, d_out, r) in enumerate(shapes)]
    src = synth.DModelInput(520, config=84, linear=0)
    X16 = synth.encode16(src.tokens(3), dt)
    taus = [gu.calibrated_tau(L, src, s) for L, s in zip(Ls, (0.4, 0.5, 0.7))]
    for widths in ((64, 64, 64), (64, 0, 32)):
        layers = [gu.prepare(L, t, max_batch=3, out_dtype=rs.F32, strip_cols=w) for L, t, w in zip(Ls, taus, widths)]
        Xd = gu.to_dev16(X16)
        for B in (1, 3):
            Ys = [gu._alloc_out(l, B) for l in layers]
            rs.rsparse_linear_group(layers, Xd.data_ptr(), B, [y.data_ptr() for y in Ys], gu.stream_ptr())
            torch.cuda.synchronize()
            for L, t, l, y in zip(Ls, taus, layers, Ys):
                want = gu.oracle_linear(L, X16[:B], t)
                gu.check_outputs(y.cpu().numpy().astype(np.float64), want["Y"], rs.F32)
                got = {"act": [rs.rsparse_last_active(l, b) for b in range(B)], "union": rs.rsparse_last_active(l, -1)}
                gu.check_lists(got, want)
            Yd = [gu._alloc_out(l, B) for l in layers]
            rs.rsparse_dense_ref_group(layers, Xd.data_ptr(), B, [y.data_ptr() for y in Yd], gu.stream_ptr())
            torch.cuda.synchronize()
            import oracle
            for L, y in zip(Ls, Yd):
                gu.check_outputs(y.cpu().numpy().astype(np.float64), oracle.dense_linear(L.W16, X16[:B], dt, dt), rs.F32)
        for l in layers:
            l.destroy()


def test_gated_mlp_entry_points_on_strip_layers(ragged):
    """rsparse_mlp_gate_up and rsparse_linear_gated on strip layers (the activation runs as a launch of its own)."""
    import oracle
    torch = gu.torch_mod()
    dt = synth.BF16
    gate = synth.make_layer(264, 520, 16, dt, config=85, linear=0)
    up = synth.make_layer(264, 520, 16, dt, config=85, linear=1)
    down = synth.make_layer(520, 264, 16, dt, config=85, linear=2)
    src = synth.DModelInput(264, config=85, linear=0)
    X16 = synth.encode16(src.tokens(2), dt)
    tg, tu = gu.calibrated_tau(gate, src, 0.5), gu.calibrated_tau(up, src, 0.5)
    lg, lu = (gu.prepare(L, t, max_batch=2, strip_cols=32) for L, t in ((gate, tg), (up, tu)))
    Xd = gu.to_dev16(X16)
    H = torch.zeros((2, 520), dtype=torch.int16, device="cuda")
    rs.rsparse_mlp_gate_up(lg, lu, Xd.data_ptr(), 2, H.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    wg, wu = gu.oracle_linear(gate, X16, tg), gu.oracle_linear(up, X16, tu)
    h_want = synth.decode16(oracle.gated_input(synth.encode16(wg["Y"], dt), synth.encode16(wu["Y"], dt), dt), dt)
    h_got = synth.decode16(H.cpu().numpy().view(np.uint16), dt)
    assert np.linalg.norm(h_got - h_want) <= 1e-2 * np.linalg.norm(h_want)       # g, u each within a rounding step
    # down projection on the gated input formed on the device
    G16, U16 = synth.encode16(wg["Y"], dt), synth.encode16(wu["Y"], dt)
    Xh = oracle.gated_input(G16, U16, dt)
    td = oracle.quantile_tau(Xh, dt, 0.5)
    ld = gu.prepare(down, td, max_batch=2, out_dtype=rs.F32, strip_cols=64)
    Y = gu._alloc_out(ld, 2)
    Gd, Ud = gu.to_dev16(G16), gu.to_dev16(U16)          # (kept alive until the call has run)
    rs.rsparse_linear_gated(ld, Gd.data_ptr(), Ud.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    want = gu.oracle_linear(down, Xh, td)
    gu.check_outputs(Y.cpu().numpy().astype(np.float64), want["Y"], rs.F32)
    got = {"act": [rs.rsparse_last_active(ld, b) for b in range(2)], "union": rs.rsparse_last_active(ld, -1)}
    gu.check_lists(got, want)
    for l in (lg, lu, ld):
        l.destroy()


def test_config0_full_size():
    """configs[0] (4096 x 4096 fp16, r = 256, 50 %) at the strip kernel's default launch shape."""
    L = synth.make_layer(4096, 4096, 256, synth.F16, config=0, linear=0)
    src = synth.DModelInput(L.d_in, config=0, linear=0)
    tau = gu.calibrated_tau(L, src, 0.5)
    X16 = synth.encode16(src.tokens(2), L.dtype)
    for W in (64, 128):
        for b in range(2):
            got, _ = _parity(L, X16[b], tau, W)
            assert abs(len(got["act"][0]) - 2048) < 200


def test_argument_checks():
    L = synth.make_layer(264, 264, 8, synth.F16, config=86, linear=0)
    with pytest.raises(rs.RSparseError):
        gu.prepare(L, 0.5, strip_cols=48)
    Q, S, Z = synth.quantize_q4(synth.decode16(L.W16, L.dtype)[:, :256], L.dtype, 128)
    with pytest.raises(rs.RSparseError):
        rs.rsparse_prepare_q4(rs.make_config(256, 264, 0, 0.5, L.dtype, strip_cols=64), Q, S, Z, 128)
