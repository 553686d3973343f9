"""GPU parity of the layer on 4-bit weights (Sec. 4.4: R-Sparse combined with 4-bit GPTQ weights): the HIP
path through the C ABI against the fp64 oracle, which dequantises W~ = s (q - z) exactly and applies the
plain layer.  Kept-channel lists must be equal; outputs within the tolerances of the 16-bit path (the
kernel's fp32 sums per quantisation group add one rounding per group, far inside them)."""
import numpy as np
import pytest

import oracle
import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu
INF = float("inf")


class Q4Layer:
    def __init__(self, L, group):
        self.L, self.group = L, group
        self.Q, self.S16, self.Z = synth.quantize_q4(synth.decode16(L.W16, L.dtype), L.dtype, group)

    def prepare(self, tau, max_batch=1, out_dtype=None, **kw):
        L = self.L
        cfg = rs.make_config(L.d_in, L.d_out, L.rank, tau, L.dtype, max_batch=max_batch, out_dtype=out_dtype, **kw)
        return rs.rsparse_prepare_q4(cfg, self.Q, self.S16, self.Z, self.group, L.U16 if L.rank else None,
                                     L.SV16 if L.rank else None)

    def oracle(self, X16, tau, **kw):
        L = self.L
        return oracle.rsparse_linear_q4(self.Q, self.S16, self.Z, L.U16 if L.rank else None,
                                        L.SV16 if L.rank else None, np.atleast_2d(X16), L.dtype, tau,
                                        group=self.group, nthreads=8, **kw)

    def dense(self, X16):
        W = oracle.dequant_q4(self.Q, self.S16, self.Z, self.L.dtype, self.group)
        return oracle.dense_linear(W, np.atleast_2d(X16), oracle.F64, self.L.dtype, nthreads=8)


@pytest.fixture(scope="module")
def ragged_q4():
    """Three 1024-column tiles with a ragged tail (2120 = 2 * 1024 + 72), nine groups of 128."""
    return {dt: Q4Layer(synth.make_layer(1152, 2120, 40, dt, config=91, linear=dt), 128)
            for dt in (synth.F16, synth.BF16)}


def _parity(q, X16, tau, out_dtype=None, tuning=None, **kw):
    X16 = np.atleast_2d(X16)
    layer = q.prepare(tau, max_batch=X16.shape[0], out_dtype=out_dtype, **kw)
    if tuning:
        rs.rsparse_set_tuning(layer, **tuning)
    got = gu.run_linear(layer, X16)
    want = q.oracle(X16, tau, cmp_mode=kw.get("cmp_mode", 0), batch_mask_mode=kw.get("batch_mask_mode", 0))
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
    layer.destroy()
    return got, want


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
@pytest.mark.parametrize("out", [None, rs.F32])
def test_q4_ragged_batch1(ragged_q4, dt, out):
    q = ragged_q4[dt]
    X16, src = gu.tokens_for(q.L, 2, linear=dt)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    for b in range(2):
        got, _ = _parity(q, X16[b], tau, out_dtype=out)
        assert 0.3 * q.L.d_in < len(got["act"][0]) < 0.7 * q.L.d_in


@pytest.mark.parametrize("B", [2, 3, 4, 5, 8, 9, 16, 17, 32])
@pytest.mark.parametrize("mask_mode", [0, 1])
def test_q4_batches(ragged_q4, B, mask_mode):
    """Up to 4 tokens share one pass over the codes; larger batches run as batch tiles of 4.  Both launch
    forms (the one-launch form covers up to 16 tokens and falls back to two launches beyond)."""
    q = ragged_q4[synth.BF16]
    X16, src = gu.tokens_for(q.L, B, linear=B)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    _parity(q, X16, tau, out_dtype=rs.F32, batch_mask_mode=mask_mode)
    _parity(q, X16, tau, batch_mask_mode=mask_mode)
    _parity(q, X16, tau, out_dtype=rs.F32, batch_mask_mode=mask_mode, tuning=dict(launches=1))


def test_q4_edge_thresholds_and_sparsities(ragged_q4):
    q = ragged_q4[synth.F16]
    X16, src = gu.tokens_for(q.L, 1)
    for tau in (-INF, 0.0, INF):
        for mode in (0, 1):
            _parity(q, X16, tau, out_dtype=rs.F32, cmp_mode=mode)
    for s in (0.05, 0.9, 0.99):          # nearly dense, sparse, a handful of channels (most groups empty)
        _parity(q, X16, gu.calibrated_tau(q.L, src, s), out_dtype=rs.F32)


@pytest.mark.parametrize("tuning", [
    dict(splits=1, waves=1), dict(splits=1, waves=8), dict(splits=3, waves=2), dict(splits=40, waves=4),
    dict(splits=144, waves=1), dict(waves=8, lowrank_rows=1), dict(waves=2, lowrank_rows=8),
    dict(nontemporal=2), dict(splits=7, waves=8, lowrank_rows=32),
])
def test_q4_launch_shapes(ragged_q4, tuning):
    q = ragged_q4[synth.BF16]
    X16, src = gu.tokens_for(q.L, 3, linear=7)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    _parity(q, X16, tau, out_dtype=rs.F32, tuning=tuning)                       # two launches (the default)
    _parity(q, X16, tau, out_dtype=rs.F32, tuning=dict(tuning, launches=1))     # the whole layer in one launch


@pytest.mark.parametrize("group,d_in", [(32, 1056), (64, 1088), (256, 1280), (1024, 2048)])
def test_q4_group_sizes(group, d_in):
    q = Q4Layer(synth.make_layer(d_in, 1032, 16, synth.F16, config=92, linear=group), group)
    X16, src = gu.tokens_for(q.L, 2, linear=group)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    _parity(q, X16, tau, out_dtype=rs.F32)


def test_q4_rank_zero_small_and_narrow():
    q = Q4Layer(synth.make_layer(128, 8, 0, synth.BF16, config=93, linear=0), 128)     # one group, one lane
    X16, src = gu.tokens_for(q.L, 4)
    _parity(q, X16, gu.calibrated_tau(q.L, src, 0.5), out_dtype=rs.F32)
    q = Q4Layer(synth.make_layer(256, 520, 0, synth.F16, config=93, linear=1), 128)
    X16, src = gu.tokens_for(q.L, 1)
    _parity(q, X16, gu.calibrated_tau(q.L, src, 0.5))


def test_q4_extreme_codes_and_zero_points():
    """All-0 and all-15 codes against zero points 15 and 0: the largest cancellation between the two
    per-group sums the kernel keeps."""
    L = synth.make_layer(512, 1032, 8, synth.F16, config=94, linear=0)
    q = Q4Layer(L, 128)
    rng = np.random.default_rng(3)
    q.Q = np.where(rng.random(q.Q.shape) < 0.5, 0, 15).astype(np.uint8)
    q.Z = np.where(rng.random(q.Z.shape) < 0.5, 0, 15).astype(np.uint8)
    X16, src = gu.tokens_for(L, 2)
    _parity(q, X16, gu.calibrated_tau(L, src, 0.5), out_dtype=rs.F32)


@pytest.mark.parametrize("launches", [1, 2])
@pytest.mark.parametrize("B", [1, 4])
def test_q4_both_launch_forms_on_a_reused_handle(ragged_q4, launches, B):
    """Back-to-back calls with different kept sets on one handle, in either form: the one-launch form's arrival
    counters, published intermediates and accumulators must be back in their idle state after every call."""
    q = ragged_q4[synth.F16]
    X16, src = gu.tokens_for(q.L, B, linear=60 + B)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    layer = q.prepare(tau, max_batch=B, out_dtype=rs.F32)
    rs.rsparse_set_tuning(layer, launches=launches)
    for t in (tau, -INF, gu.calibrated_tau(q.L, src, 0.8), INF, tau):
        rs.rsparse_set_tau(layer, t)
        got = gu.run_linear(layer, X16)
        rs.rsparse_synchronize(layer)
        want = q.oracle(X16, t)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


def test_q4_bounded_wait_runs_out_and_the_handle_recovers(ragged_q4):
    """The error path of the one-launch form, forced from the host (stage 1 publishes nothing, the wait bound is
    a few polls): every kernel still ends, the call is reported invalid, the next call is correct again."""
    q = ragged_q4[synth.BF16]
    X16, src = gu.tokens_for(q.L, 2, linear=78)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    layer = q.prepare(tau, max_batch=2, out_dtype=rs.F32)
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
        want = q.oracle(X16, tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
    layer.destroy()


def test_q4_dense_baseline_and_reuse(ragged_q4):
    q = ragged_q4[synth.F16]
    X16, src = gu.tokens_for(q.L, 4, linear=3)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    layer = q.prepare(tau, max_batch=4, out_dtype=rs.F32)
    for B in (4, 1, 3, 2):
        got = gu.run_linear(layer, X16[:B])
        want = q.oracle(X16[:B], tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], rs.F32)
        gu.check_outputs(gu.run_dense(layer, X16[:B]), q.dense(X16[:B]), rs.F32)
    rs.rsparse_set_tau(layer, 0.0)
    gu.check_outputs(gu.run_linear(layer, X16[:2], lists=False)["Y"], q.oracle(X16[:2], 0.0)["Y"], rs.F32)
    assert rs.rsparse_required_bytes(layer, 1, q.L.d_in) > rs.rsparse_dense_bytes(layer, 1)
    layer.destroy()


def test_q4_gated_input_and_mlp_first_half():
    """The other entry points accept such layers: the gated input (Sec. 3.1) ahead of a 4-bit down projection, and
    gate / up with 4-bit weights followed by the activation."""
    torch = gu.torch_mod()
    dt = synth.BF16
    down = Q4Layer(synth.make_layer(1152, 520, 16, dt, config=95, linear=0), 128)
    g, u = synth.GateUpPair(1152, config=95, linear=0).tokens(2)
    G16, U16 = synth.encode16(g, dt), synth.encode16(u, dt)
    x16 = oracle.gated_input(G16, U16, dt)
    tau = oracle.quantile_tau(x16, dt, 0.5)
    layer = down.prepare(tau, max_batch=2, out_dtype=rs.F32)
    Gd, Ud = gu.to_dev16(G16), gu.to_dev16(U16)
    Y = torch.zeros((2, 520), dtype=torch.float32, device="cuda")
    rs.rsparse_linear_gated(layer, Gd.data_ptr(), Ud.data_ptr(), 2, Y.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    want = down.oracle(x16, tau)
    gu.check_outputs(Y.cpu().numpy().astype(np.float64), want["Y"], rs.F32)
    assert np.array_equal(rs.rsparse_last_active(layer, 1), want["act"][1])
    layer.destroy()

    gate = Q4Layer(synth.make_layer(640, 1032, 16, dt, config=95, linear=1), 128)
    up = Q4Layer(synth.make_layer(640, 1032, 16, dt, config=95, linear=2), 128)
    X16, src = gu.tokens_for(gate.L, 2, linear=5)
    tau = gu.calibrated_tau(gate.L, src, 0.5)
    lg, lu = gate.prepare(tau, max_batch=2), up.prepare(tau, max_batch=2)
    Xd = gu.to_dev16(X16)
    H = torch.zeros((2, 1032), dtype=torch.int16, device="cuda")
    rs.rsparse_mlp_gate_up(lg, lu, Xd.data_ptr(), 2, H.data_ptr(), gu.stream_ptr())
    torch.cuda.synchronize()
    got = synth.decode16(H.cpu().numpy().view(np.uint16), dt)
    yg, yu = gate.oracle(X16, tau)["Y"], up.oracle(X16, tau)["Y"]
    want = synth.decode16(oracle.gated_input(synth.encode16(yg, dt), synth.encode16(yu, dt), dt), dt)
    # g and u are rounded to 16 bits before the activation on both sides; a last-bit difference in either
    # moves the product by one 16-bit step, so compare with the 16-bit tolerances
    gu.check_outputs(got, want, dt)
    lg.destroy()
    lu.destroy()


def test_q4_mixed_group_call(ragged_q4):
    """A grouped call may mix 4-bit and 16-bit layers that read the same input."""
    torch = gu.torch_mod()
    q = ragged_q4[synth.BF16]
    L16 = synth.make_layer(1152, 520, 24, synth.BF16, config=96, linear=0)
    X16, src = gu.tokens_for(q.L, 2, linear=9)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    a = q.prepare(tau, max_batch=2, out_dtype=rs.F32)
    b = gu.prepare(L16, tau, max_batch=2, out_dtype=rs.F32)
    Xd = gu.to_dev16(X16)
    Ya = torch.zeros((2, q.L.d_out), dtype=torch.float32, device="cuda")
    Yb = torch.zeros((2, L16.d_out), dtype=torch.float32, device="cuda")
    rs.rsparse_linear_group([a, b], Xd.data_ptr(), 2, [Ya.data_ptr(), Yb.data_ptr()], gu.stream_ptr())
    torch.cuda.synchronize()
    gu.check_outputs(Ya.cpu().numpy().astype(np.float64), q.oracle(X16, tau)["Y"], rs.F32)
    gu.check_outputs(Yb.cpu().numpy().astype(np.float64), gu.oracle_linear(L16, X16, tau)["Y"], rs.F32)
    a.destroy()
    b.destroy()


def test_q4_config1_shapes_as_benchmarked():
    """The MLP shapes of the benchmark workload (4096 -> 11008 and 11008 -> 4096, bf16, r = 512 and the small
    rank of a sparse-heavy recipe) at the default launch shape, captured into a HIP graph and replayed, both
    launch forms; every output of every replay against the oracle."""
    torch = gu.torch_mod()
    dt = synth.BF16
    for d_in, d_out, rank, kind in ((4096, 11008, 512, "dmodel"), (11008, 4096, 64, "down")):
        L = synth.random_layer(d_in, d_out, rank, dt, seed=4100 + rank)
        q = Q4Layer(L, 128)
        X16, src = gu.tokens_for(L, 1, kind=kind, linear=rank)
        tau = gu.calibrated_tau(L, src, 0.5)
        layer = q.prepare(tau, max_batch=1)
        want = q.oracle(X16, tau)
        Xd = gu.to_dev16(X16)
        Y = gu._alloc_out(layer, 1)
        for launches in (1, 2):
            rs.rsparse_set_tuning(layer, launches=launches)
            got = gu.run_linear(layer, X16)
            gu.check_lists(got, want)
            gu.check_outputs(got["Y"], want["Y"], dt)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                rs.rsparse_linear(layer, Xd.data_ptr(), 1, Y.data_ptr(), torch.cuda.current_stream().cuda_stream)
            for rep in range(3):
                Y.fill_(0x7FFF)
                graph.replay()
                torch.cuda.synchronize()
                rs.rsparse_synchronize(layer)
                gu.check_outputs(gu._read_out(layer, Y), want["Y"], dt)
        gu.check_outputs(gu.run_dense(layer, X16), q.dense(X16), dt)
        layer.destroy()


@pytest.mark.parametrize("seed", range(4))
def test_q4_random_shapes_and_settings(seed):
    """Seeded sweep over small random layers on 4-bit weights: group sizes 32-256, d_in any multiple of the
    group, d_out any multiple of 8 (1-3 column tiles, ragged), ranks from 0 up, 1-32 tokens, both dtypes, compare
    modes, mask modes and launch forms, random launch shapes.  Lists equal, outputs within the fp32-output bound."""
    rng = np.random.default_rng(4321 + seed)
    for case in range(8):
        group = int(rng.choice([32, 64, 128, 256]))
        d_in = group * int(rng.integers(1, max(2, 1400 // group)))
        d_out = 8 * int(rng.integers(1, 330))
        rank = 8 * int(rng.integers(0, min(min(d_in, d_out) // 8, 12) + 1))
        dt = int(rng.integers(0, 2))
        B = int(rng.choice([1, 1, 2, 3, 4, 4, 5, 7, 12, 16, 17, 32]))
        cmp_mode, mask_mode = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        q = Q4Layer(synth.random_layer(d_in, d_out, rank, dt, seed=9500 + 100 * seed + case), group)
        src = synth.DModelInput(d_in, config=89, linear=10 * seed + case)
        X16 = synth.encode16(src.tokens(B), dt)
        s_level = float(rng.choice([0.0, 0.3, 0.5, 0.5, 0.8, 0.97, 1.0]))
        tau = gu.calibrated_tau(q.L, src, s_level) if 0.0 < s_level < 1.0 else (-INF if s_level == 0.0 else INF)
        tuning = {"launches": int(rng.integers(1, 3))}
        if rng.random() < 0.5:
            tuning.update(splits=int(rng.integers(1, 40)), waves=int(rng.choice([1, 2, 4, 8])))
        if rng.random() < 0.3:
            tuning.update(lowrank_rows=int(rng.integers(1, 33)))
        print("case", dict(group=group, d_in=d_in, d_out=d_out, rank=rank, dt=dt, B=B, cmp=cmp_mode, mask=mask_mode,
                           s=s_level, **tuning), flush=True)
        _parity(q, X16, tau, out_dtype=rs.F32, tuning=tuning, cmp_mode=cmp_mode, batch_mask_mode=mask_mode)


@pytest.mark.parametrize("dt", [synth.F16, synth.BF16])
def test_q4_dense_rowdot_over_row_major_codes(ragged_q4, dt):
    """The row-dot dense baseline (dense_rowmajor = 1): every batch tile, both output types, extreme codes, and the same
    result as the channel-major dense form; R-Sparse on the same handle is untouched by the extra copy."""
    q = ragged_q4[dt]
    X16, src = gu.tokens_for(q.L, 9, kind="dmodel", config=91)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    for out_dtype in (None, rs.F32):
        layer = q.prepare(tau, max_batch=9, out_dtype=out_dtype, dense_rowmajor=1)
        for B in (1, 2, 3, 4, 9):
            want = q.dense(X16[:B])
            gu.check_outputs(gu.run_dense(layer, X16[:B]), want, layer.cfg.out_dtype)          # row-dot (default with the copy)
            rs.rsparse_set_tuning(layer, dense_kernel=1)
            gu.check_outputs(gu.run_dense(layer, X16[:B]), want, layer.cfg.out_dtype)          # channel-major, every channel kept
            rs.rsparse_set_tuning(layer)
        got = gu.run_linear(layer, X16[:2])
        want = q.oracle(X16[:2], tau)
        gu.check_lists(got, want)
        gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
        layer.destroy()
    # without the copy the row-dot form is refused, not silently replaced
    layer = q.prepare(tau, max_batch=1)
    rs.rsparse_set_tuning(layer, dense_kernel=2)
    with pytest.raises(rs.RSparseError):
        gu.run_dense(layer, X16[:1])
    layer.destroy()


def test_q4_dense_rowdot_extreme_codes_group_sizes_and_benchmark_shape():
    dt = synth.BF16
    for group, d_in in ((32, 256), (1024, 2048), (128, 4096)):
        L = synth.make_layer(d_in, 264, 0, dt, config=93, linear=group % 7)
        q = Q4Layer(L, group)
        q.Q[:8, :] = 15
        q.Z[:8, :] = 0
        q.Q[8:16, :] = 0
        q.Z[8:16, :] = 15
        X16, _ = gu.tokens_for(L, 2, config=93)
        layer = q.prepare(0.0, max_batch=2, out_dtype=rs.F32, dense_rowmajor=1)
        gu.check_outputs(gu.run_dense(layer, X16), q.dense(X16), rs.F32)
        layer.destroy()
    L = synth.random_layer(11008, 4096, 64, dt, seed=17)
    q = Q4Layer(L, 128)
    X16, _ = gu.tokens_for(L, 1, kind="down", config=93)
    layer = q.prepare(0.0, max_batch=1, dense_rowmajor=1)
    gu.check_outputs(gu.run_dense(layer, X16), q.dense(X16), dt)
    layer.destroy()


@pytest.mark.parametrize("launches", [1, 2])
def test_q4_nan_inf_and_negative_zero_inputs(ragged_q4, launches):
    """NaN is never kept and reaches every output through the low-rank part; -0 is 0; a kept +-Inf channel makes that
    token's outputs non-finite (NaN here, where the definition W~ x gives +-Inf or NaN output by output -- the
    documented deviation of the factored group sums)."""
    dt = synth.BF16
    q = ragged_q4[dt]
    X16, src = gu.tokens_for(q.L, 4, config=91)
    tau = gu.calibrated_tau(q.L, src, 0.5)
    x = synth.decode16(X16, dt)
    x[0, 5] = np.nan
    x[1, 7] = -0.0
    x[1, 8] = 0.0
    x[2, 9] = np.inf
    x[3, 11] = -np.inf
    X16 = synth.encode16(x, dt)
    layer = q.prepare(tau, max_batch=4, out_dtype=rs.F32)
    rs.rsparse_set_tuning(layer, launches=launches)
    got = gu.run_linear(layer, X16)
    want = q.oracle(X16, tau)
    gu.check_lists(got, want)
    assert np.all(np.isnan(got["Y"][0])) and np.all(np.isnan(want["Y"][0]))
    gu.check_outputs(got["Y"][1:2], want["Y"][1:2], rs.F32)
    for b in (2, 3):
        assert not np.any(np.isfinite(want["Y"][b]))                  # the definition: +-Inf, or NaN where W~[o][c] = 0
        assert np.all(~np.isfinite(got["Y"][b]))
    layer.destroy()
