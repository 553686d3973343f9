"""GPU parity at the full sizes of the benchmark configurations that the small ragged layers do not reach: the
launch shapes (channel splits, 8-token register tiles with 4-wave workgroups, K slices of the matrix-core kernels,
strips) differ at these sizes.  Operands are i.i.d. values of the workloads' scales (kernel parity does not depend on
W being an SVD product); every output of every token is compared with the fp64 oracle, kept lists must be equal."""
import numpy as np
import pytest

import oracle
import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _case(d_in, d_out, rank, kind, B, seed, s=0.5, rowmajor=0, strip_cols=0, tuning=None, out_dtype=None):
    dt = synth.BF16
    L = synth.random_layer(d_in, d_out, rank, dt, seed=seed)
    src = (synth.DModelInput if kind == "dmodel" else synth.DownInput)(d_in, config=70, linear=seed % 7)
    tau = gu.calibrated_tau(L, src, s)
    X16 = synth.encode16(src.tokens(B, offset=11), dt)
    layer = gu.prepare(L, tau, max_batch=B, out_dtype=out_dtype, dense_rowmajor=rowmajor, strip_cols=strip_cols)
    if tuning:
        rs.rsparse_set_tuning(layer, **tuning)
    got = gu.run_linear(layer, X16)
    rs.rsparse_synchronize(layer)
    want = gu.oracle_linear(L, X16, tau)
    gu.check_lists(got, want)
    gu.check_outputs(got["Y"], want["Y"], layer.cfg.out_dtype)
    layer.destroy()
    return got


@pytest.mark.parametrize("B", [2, 4, 8])
@pytest.mark.parametrize("launches", [1, 2])
def test_config2_qkv_grouped_and_down(B, launches):
    """configs[2]: q / k / v (4096 x 4096, r = 256) in one grouped call and the down projection (11008 -> 4096) at
    2, 4 and 8 tokens on the vector path, both launch forms."""
    torch = gu.torch_mod()
    dt = synth.BF16
    src = synth.DModelInput(4096, config=72, linear=0)
    X16 = synth.encode16(src.tokens(B, offset=5), dt)
    Ls = [synth.random_layer(4096, 4096, 256, dt, seed=720 + i) for i in range(3)]
    taus = [gu.calibrated_tau(L, src, 0.5) for L in Ls]
    layers = [gu.prepare(L, t, max_batch=B) for L, t in zip(Ls, taus)]
    for l in layers:
        rs.rsparse_set_tuning(l, launches=launches, mfma_min_batch=33)
    Xd = gu.to_dev16(X16)
    Ys = [gu._alloc_out(l, B) for l in layers]
    rs.rsparse_linear_group(layers, Xd.data_ptr(), B, [y.data_ptr() for y in Ys], gu.stream_ptr())
    torch.cuda.synchronize()
    for L, t, l, y in zip(Ls, taus, layers, Ys):
        want = gu.oracle_linear(L, X16, t)
        gu.check_outputs(gu._read_out(l, y), want["Y"], l.cfg.out_dtype)
        got = {"act": [rs.rsparse_last_active(l, b) for b in range(B)], "union": rs.rsparse_last_active(l, -1)}
        gu.check_lists(got, want)
        l.destroy()
    _case(11008, 4096, 256, "down", B, seed=725, tuning=dict(launches=launches, mfma_min_batch=33))


@pytest.mark.parametrize("shape", [(4096, 14336, "dmodel"), (14336, 4096, "down")])
@pytest.mark.parametrize("B,rowmajor", [(1, 0), (16, 1), (16, 0)])
def test_config3_mlp_shapes(shape, B, rowmajor):
    """configs[3]: 4096 -> 14336 and 14336 -> 4096, r = 256, at 1 and 16 tokens (16 tokens: on the matrix cores with
    the row-major copy of W, in two batch tiles of 8 on the vector ALU without it), 60 % sparsity at one token."""
    d_in, d_out, kind = shape
    _case(d_in, d_out, 256, kind, B, seed=730 + B, s=0.6 if B == 1 else 0.5, rowmajor=rowmajor)


def test_config3_gqa_kv_ranks():
    """configs[3]: the skinny k / v projection 4096 -> 1024 at ranks 128 and 512, 1 and 16 tokens."""
    for rank in (128, 512):
        _case(4096, 1024, rank, "dmodel", 1, seed=740 + rank)
        _case(4096, 1024, rank, "dmodel", 16, seed=741 + rank, rowmajor=1)


@pytest.mark.parametrize("B,rowmajor", [(8, 1), (8, 0), (32, 1)])
def test_config4_gate_up(B, rowmajor):
    """configs[4]: 8192 -> 28672, r = 1024, at 8 tokens (matrix cores, and the 8-token vector kernel) and 32."""
    _case(8192, 28672, 1024, "dmodel", B, seed=750 + B, rowmajor=rowmajor)


def test_config4_down_and_kv():
    """configs[4]: 28672 -> 8192 at 32 tokens, 8192 -> 1024 with r = 1024 (the low-rank factors outweigh W) at 1."""
    _case(28672, 8192, 1024, "down", 32, seed=760, rowmajor=1)
    _case(8192, 1024, 1024, "dmodel", 1, seed=761)


@pytest.mark.parametrize("shape", [(4096, 4096, 256, "dmodel", 128), (11008, 4096, 512, "down", 64),
                                   (4096, 11008, 512, "dmodel", 128), (8192, 28672, 1024, "dmodel", 256),
                                   (28672, 8192, 1024, "down", 64)])
def test_strip_layout_at_benchmark_shapes(shape):
    """The strip kernel at the benchmark's one-token shapes and default launch shapes."""
    d_in, d_out, rank, kind, W = shape
    _case(d_in, d_out, rank, kind, 1, seed=770 + W, strip_cols=W)
    _case(d_in, d_out, rank, kind, 4, seed=771 + W, strip_cols=W, out_dtype=rs.F32)


@pytest.mark.parametrize("strip_cols", [0, 128])
def test_the_widest_input_the_library_accepts(strip_cols):
    """d_in = 65536 is the documented maximum (the token scan's LDS): one and three tokens, threshold and fixed-count
    activation, on both layouts; one more channel group is rejected on the host."""
    dt = synth.BF16
    L = synth.random_layer(65536, 264, 16, dt, seed=31)
    X16, src = gu.tokens_for(L, 3)
    tau = gu.calibrated_tau(L, src, 0.5)
    for kw, okw in ((dict(), dict()), (dict(topk=30000), dict(topk=30000))):
        layer = gu.prepare(L, tau, max_batch=4, strip_cols=strip_cols, **kw)
        for B in (1, 3):
            want = gu.oracle_linear(L, X16[:B], tau, **okw)
            got = gu.run_linear(layer, X16[:B])
            gu.check_lists(got, want)
            gu.check_outputs(got["Y"], want["Y"], dt)
        gu.check_outputs(gu.run_dense(layer, X16[:1]), oracle.dense_linear(L.W16, X16[:1], dt, dt, nthreads=8), dt)
        layer.destroy()
    if strip_cols == 0:
        # stage 1 over the channel-major copy of S_r V_r^T: default and extreme numbers of stage-1 workgroups (one would
        # need a list of 65536 entries: the library raises the count until a workgroup's list fits its LDS)
        layer = gu.prepare(L, tau, lowrank_channel_major=1)
        want = gu.oracle_linear(L, X16[:1], tau)
        for wgs in (0, 1, 8192):
            rs.rsparse_set_tuning(layer, lowrank_wgs=wgs)
            got = gu.run_linear(layer, X16[:1])
            rs.rsparse_synchronize(layer)
            gu.check_lists(got, want)
            gu.check_outputs(got["Y"], want["Y"], dt)
        layer.destroy()
    with pytest.raises(rs.RSparseError):
        rs.rsparse_prepare_factors(rs.make_config(65536 + 8, 264, 0, tau, dt), np.zeros((264, 65544), dtype=np.uint16), None, None)
