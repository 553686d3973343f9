"""GPU parity for the stage 1 that reads a channel-major copy of S_r V_r^T (config lowrank_channel_major = 1): up to
four tokens the one-launch column-tile kernel forms t from the rows of the dropped channels only (Sec. 3.4: the
low-rank part acts on x - sigma_t(x)).  Same oracle, same tolerances, kept lists bit-exact; every other path of a layer
prepared this way (more tokens, two launches, the dense reference) reads the row-major copy and must be unchanged.
Left to itself the library uses the copy only in launches of 2^26 weights or more and at four tokens under the union mask;
the small layers here force it with an explicit number of stage-1 workgroups."""
import numpy as np
import pytest

import oracle
import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
INF = float("inf")


def _layer(d_in, d_out, rank, dt, seed=0):
    return synth.make_layer(d_in, d_out, rank, dt, config=90 + seed, linear=seed)


def _check(L, layer, X16, tau, **okw):
    got = gu.run_linear(layer, X16)
    rs.rsparse_synchronize(layer)
    want = gu.oracle_linear(L, X16, tau, **okw)
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
    return got


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("rank", [8, 264, 520])
def test_one_token_against_the_oracle(dt, rank):
    """Ranks below, at and above one 512-column part (520 = one part and 8 columns), both output types, thresholds
    from 'keep everything' (no row read) to 'keep nothing' (every row read), all compare modes, several numbers of
    stage-1 workgroups incl. one per 8 channels, calls repeated on one handle (sums and counters go back to zero)."""
    L = _layer(1032, 1096, rank, dt)
    X16, src = gu.tokens_for(L, 4, linear=3)
    tau50 = gu.calibrated_tau(L, src, 0.5)
    for out in (None, rs.F32):
        for tau, cmp_mode in ((tau50, 0), (tau50, 1), (0.05, 2), (-INF, 0), (INF, 0), (gu.calibrated_tau(L, src, 0.9), 0)):
            layer = gu.prepare(L, tau, out_dtype=out, cmp_mode=cmp_mode, lowrank_channel_major=1)
            for wgs in (0, 1, 3, 129, 4096):
                rs.rsparse_set_tuning(layer, lowrank_wgs=wgs)
                for b in range(2):
                    _check(L, layer, X16[b], tau, cmp_mode=cmp_mode)
            layer.destroy()


def test_special_values_and_ties_at_the_threshold():
    dt = synth.F16
    L = _layer(1032, 520, 64, dt, seed=1)
    X16, src = gu.tokens_for(L, 1)
    tau = gu.calibrated_tau(L, src, 0.5)
    X = X16[0].copy()
    X[5], X[77], X[8] = 0x7C00, 0xFC00, 0x8000                        # +inf and -inf are kept, -0 is dropped
    X[100:110] = synth.encode16(np.full(10, tau), dt)                 # ties at the threshold
    layer = gu.prepare(L, tau, out_dtype=rs.F32, lowrank_channel_major=1)
    rs.rsparse_set_tuning(layer, lowrank_wgs=16)          # (a launch this small uses the row-major copy unless told to)
    got = _check(L, layer, X, tau)
    assert 5 in got["act"][0] and 77 in got["act"][0] and 8 not in got["act"][0]
    X[9] = 0x7E00                                                      # a NaN is dropped and poisons t
    got = _check(L, layer, X, tau)
    assert 9 not in got["act"][0] and np.all(np.isnan(got["Y"]))
    X[9] = 0
    _check(L, layer, X, tau)                                           # and the handle is clean again
    layer.destroy()


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("mask_mode", [0, 1, 2])
def test_two_to_four_tokens(dt, mask_mode):
    """Batch tiles of 2 and 4 tokens: a channel's row is read if any token of the tile drops it, every token with its
    own coefficient (zero where it keeps the channel); with the union mask the dropped channels are the few that no
    token of the batch keeps.  Ragged tiles (3 tokens), a token of all zeros, repeated calls."""
    L = _layer(1032, 1096, 520, dt, seed=10)
    X16, src = gu.tokens_for(L, 8, linear=5)
    X16[2, :] = 0                                                      # a token that keeps nothing at tau > 0
    tau = gu.calibrated_tau(L, src, 0.5)
    for out in (None, rs.F32):
        layer = gu.prepare(L, tau, max_batch=4, out_dtype=out, batch_mask_mode=mask_mode, lowrank_channel_major=1)
        for wgs in (0, 5, 129):
            rs.rsparse_set_tuning(layer, lowrank_wgs=wgs)
            for B in (2, 3, 4, 1):
                _check(L, layer, X16[:B], tau, batch_mask_mode=1 if (mask_mode == 1 or (mask_mode == 2 and B >= 4)) else 0)
        layer.destroy()
    # fixed-count activation with a bias at three tokens
    bias = np.random.Generator(np.random.PCG64(9)).standard_normal(1096).astype(np.float32)
    layer = gu.prepare(L, 0.0, max_batch=4, out_dtype=rs.F32, topk=400, lowrank_channel_major=1)
    rs.rsparse_set_tuning(layer, lowrank_wgs=20)
    rs.rsparse_set_bias(layer, bias)
    _check(L, layer, X16[3:6], 0.0, topk=400, bias=bias.astype(np.float64))
    layer.destroy()


def test_other_paths_of_such_a_layer_are_unchanged():
    """More than four tokens, the two-launch form, a workgroup too narrow for the rank's parts, the entry point that
    allocates nothing and the dense reference read the row-major copy."""
    dt = synth.BF16
    L = _layer(1032, 1096, 520, dt, seed=2)
    X16, src = gu.tokens_for(L, 8)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, max_batch=8, out_dtype=rs.F32, lowrank_channel_major=1)
    for B in (1, 2, 5, 8):
        _check(L, layer, X16[:B], tau)
    for tuning in (dict(launches=2), dict(waves=1), dict(splits=3, waves=2)):
        rs.rsparse_set_tuning(layer, **tuning)
        _check(L, layer, X16[:1], tau)
    rs.rsparse_set_tuning(layer)
    gu.check_outputs(gu.run_dense(layer, X16[:1]), oracle.dense_linear(L.W16, X16[:1], dt, dt, nthreads=4), rs.F32)
    torch = gu.torch_mod()
    Xd = gu.to_dev16(X16[:1])
    Y = gu._alloc_out(layer, 1)
    rs.rsparse_linear_static(layer, Xd.data_ptr(), 1, Y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    gu.check_outputs(Y.cpu().numpy().astype(np.float64), gu.oracle_linear(L, X16[:1], tau)["Y"], rs.F32)
    layer.destroy()


def test_fixed_count_activation_bias_and_grouped_calls():
    dt = synth.BF16
    Ls = [_layer(1032, d_out, r, dt, seed=3 + i) for i, (d_out, r) in enumerate(((520, 64), (264, 0), (1096, 264)))]
    X16, src = gu.tokens_for(Ls[0], 2)
    tau = gu.calibrated_tau(Ls[0], src, 0.5)
    bias = np.random.Generator(np.random.PCG64(8)).standard_normal(520).astype(np.float32)
    # fixed-count activation with a bias
    layer = gu.prepare(Ls[0], 0.0, out_dtype=rs.F32, topk=300, lowrank_channel_major=1)
    rs.rsparse_set_tuning(layer, lowrank_wgs=12)
    rs.rsparse_set_bias(layer, bias)
    for b in range(2):
        got = _check(Ls[0], layer, X16[b], 0.0, topk=300, bias=bias.astype(np.float64))
        assert len(got["act"][0]) == 300
    layer.destroy()
    # a group whose layers differ in rank and in the flag
    torch = gu.torch_mod()
    layers = [gu.prepare(L, tau, out_dtype=rs.F32, lowrank_channel_major=flag) for L, flag in zip(Ls, (1, 1, 0))]
    for l in layers:
        rs.rsparse_set_tuning(l, lowrank_wgs=10)
    Xd = gu.to_dev16(X16[:1])
    Ys = [gu._alloc_out(l, 1) for l in layers]
    for _ in range(2):
        rs.rsparse_linear_group(layers, Xd.data_ptr(), 1, [y.data_ptr() for y in Ys], gu.stream_ptr())
        torch.cuda.synchronize()
        for L, l, y in zip(Ls, layers, Ys):
            want = gu.oracle_linear(L, X16[:1], tau)
            gu.check_outputs(y.cpu().numpy().astype(np.float64), want["Y"], rs.F32)
            assert np.array_equal(rs.rsparse_last_active(l, 0), want["act"][0])
    for l in layers:
        l.destroy()
    # gate / up with the activation in the kernel's finish
    Lg, Lu = _layer(1032, 520, 64, dt, seed=7), _layer(1032, 520, 32, dt, seed=8)
    g = gu.prepare(Lg, tau, lowrank_channel_major=1)
    u = gu.prepare(Lu, tau, lowrank_channel_major=1)
    rs.rsparse_set_tuning(g, lowrank_wgs=8)
    rs.rsparse_set_tuning(u, lowrank_wgs=24)
    H = torch.zeros((1, 520), dtype=torch.int16, device="cuda")
    rs.rsparse_mlp_gate_up(g, u, Xd.data_ptr(), 1, H.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    yg = gu.oracle_linear(Lg, X16[:1], tau)["Y"]
    yu = gu.oracle_linear(Lu, X16[:1], tau)["Y"]
    want_h = yg / (1.0 + np.exp(-yg)) * yu
    got_h = synth.decode16(H.cpu().numpy().view(np.uint16), dt)
    assert np.linalg.norm(got_h - want_h) <= 1.5e-2 * np.linalg.norm(want_h)
    g.destroy()
    u.destroy()


def test_replayed_graph_and_the_bounded_wait():
    torch = gu.torch_mod()
    dt = synth.BF16
    L = _layer(1032, 1096, 264, dt, seed=9)
    X16, src = gu.tokens_for(L, 4)
    tau = gu.calibrated_tau(L, src, 0.5)
    layer = gu.prepare(L, tau, out_dtype=rs.F32, lowrank_channel_major=1)
    rs.rsparse_set_tuning(layer, lowrank_wgs=16)
    Xd = gu.to_dev16(X16[:1])
    Y, Ye = gu._alloc_out(layer, 1), gu._alloc_out(layer, 1)
    rs.rsparse_linear(layer, Xd.data_ptr(), 1, Y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rs.rsparse_linear(layer, Xd.data_ptr(), 1, Y.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        xb = X16[rep:rep + 1]
        Xd.copy_(torch.from_numpy(np.ascontiguousarray(xb).view(np.int16)))
        Y.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = Y.cpu().numpy().astype(np.float64)
        rs.rsparse_linear(layer, Xd.data_ptr(), 1, Ye.data_ptr(), gu.stream_ptr())
        torch.cuda.synchronize()
        want = gu.oracle_linear(L, xb, tau)
        gu.check_outputs(got, want["Y"], rs.F32)
        eager = Ye.cpu().numpy().astype(np.float64)
        assert np.linalg.norm(got - eager) <= 1e-5 * np.linalg.norm(eager)
        assert np.array_equal(rs.rsparse_last_active(layer, 0), want["act"][0])
    # stage 1 publishes nothing: every bounded wait runs out, the kernel ends, the call is reported invalid, the sums
    # it left are gone (the last stage-1 workgroup swaps them out either way) and the next call is right
    rs.rsparse_set_tuning(layer, lowrank_wgs=16, debug_skip_stage1=1, debug_wait_polls=4)
    rs.rsparse_linear(layer, Xd.data_ptr(), 1, Y.data_ptr(), gu.stream_ptr())
    with pytest.raises(rs.RSparseError) as e:
        rs.rsparse_synchronize(layer)
    assert e.value.status == rs.binding.EHIP
    rs.rsparse_set_tuning(layer, lowrank_wgs=16)
    for b in range(2):
        _check(L, layer, X16[b], tau)
    layer.destroy()


def test_full_size_down_projection():
    """28672 -> 8192, r = 1024, bf16, one token at the default launch shape: every output against the oracle."""
    dt = synth.BF16
    L = synth.random_layer(28672, 8192, 1024, dt, seed=21)
    src = synth.DownInput(28672, config=4, linear=6)
    tau = rs.rsparse_calibrate_tau(synth.encode16(src.tokens(64, stream=synth.STREAM_CALIB), dt), dt, 0.5)
    X16 = synth.encode16(src.tokens(2), dt)
    layer = gu.prepare(L, tau, lowrank_channel_major=1)
    for b in range(2):
        got = _check(L, layer, X16[b], tau)
        assert abs(len(got["act"][0]) - 14336) < 1500
    layer.destroy()


@pytest.mark.parametrize("seed", list(range(4)))
def test_random_shapes_and_settings(seed):
    """Seeded sweep over small random layers with the channel-major stage 1 forced: every dimension a multiple of 8
    from 8 up, ranks from 8 to full (one to three 512-column parts, ragged), 1-4 tokens, both dtypes, all compare and
    mask modes, random launch shapes and numbers of stage-1 workgroups.  Lists equal, outputs within the fp32 bound."""
    rng = np.random.default_rng(4321 + seed)
    for case in range(8):
        d_in = 8 * int(rng.integers(1, 150))
        d_out = 8 * int(rng.integers(1, 200))
        rank = 8 * int(rng.integers(1, min(d_in, d_out) // 8 + 1))
        dt = int(rng.integers(0, 2))
        B = int(rng.choice([1, 1, 2, 3, 4]))
        cmp_mode, mask_mode = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        L = synth.random_layer(d_in, d_out, rank, dt, seed=7000 + 100 * seed + case)
        src = synth.DModelInput(d_in, config=91, linear=10 * seed + case)
        X16 = synth.encode16(src.tokens(B), dt)
        s_level = float(rng.choice([0.0, 0.3, 0.5, 0.5, 0.8, 1.0]))
        tau = gu.calibrated_tau(L, src, s_level) if 0.0 < s_level < 1.0 else (-INF if s_level == 0.0 else INF)
        if cmp_mode == 2 and not np.isfinite(tau):
            tau = 0.0
        tuning = {"lowrank_wgs": int(rng.integers(1, 200))}
        if rng.random() < 0.5:
            tuning.update(splits=int(rng.integers(1, 40)), waves=int(rng.choice([2, 4, 8])))
        label = dict(d_in=d_in, d_out=d_out, rank=rank, dt=dt, B=B, cmp=cmp_mode, mask=mask_mode, s=s_level, **tuning)
        print("case", label, flush=True)
        layer = gu.prepare(L, tau, max_batch=4, out_dtype=rs.F32, cmp_mode=cmp_mode, batch_mask_mode=mask_mode,
                           lowrank_channel_major=1)
        rs.rsparse_set_tuning(layer, **tuning)
        union = mask_mode == 1 or (mask_mode == 2 and B >= 4)
        for _ in range(2):
            _check(L, layer, X16, tau, cmp_mode=cmp_mode, batch_mask_mode=1 if union else 0)
        layer.destroy()
