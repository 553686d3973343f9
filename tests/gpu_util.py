"""Helpers for the GPU parity tests: device buffers via torch, calls through the C ABI."""
import numpy as np

import oracle
import paper_2504_19449_amd as rs
from paper_2504_19449_amd import synth

# spec tolerances for 16-bit outputs, and the fp32-output bound used to check the arithmetic
# itself: fp32 accumulation of n <= ~3e4 terms in arbitrary order has relative error
# <= ~sqrt(n) * 2^-24 ~ 1e-5 of the terms' magnitude, and ||y|| is of the terms' order here.
REL_L2_16 = 2e-3
MAX_ABS_16 = 1e-2
REL_L2_F32 = 2e-5


def torch_mod():
    import torch
    return torch


def to_dev16(bits):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def stream_ptr():
    return torch_mod().cuda.current_stream().cuda_stream


def prepare(L, tau, max_batch=1, out_dtype=None, **cfg_kw):
    cfg = rs.make_config(L.d_in, L.d_out, L.rank, tau, L.dtype, max_batch=max_batch, out_dtype=out_dtype, **cfg_kw)
    U16 = L.U16 if L.rank else None
    SV16 = L.SV16 if L.rank else None
    return rs.rsparse_prepare_factors(cfg, L.W16, U16, SV16)


def _alloc_out(layer, B):
    torch = torch_mod()
    if layer.cfg.out_dtype == rs.F32:
        return torch.full((B, layer.cfg.d_out), float("nan"), dtype=torch.float32, device="cuda")
    return torch.full((B, layer.cfg.d_out), 0x7FFF, dtype=torch.int16, device="cuda")


def _read_out(layer, Y):
    torch = torch_mod()
    torch.cuda.synchronize()
    if layer.cfg.out_dtype == rs.F32:
        return Y.cpu().numpy().astype(np.float64)
    return synth.decode16(Y.cpu().numpy().view(np.uint16), layer.cfg.out_dtype)


def run_linear(layer, X16, lists=True):
    X16 = np.atleast_2d(X16)
    B = X16.shape[0]
    Xd = to_dev16(X16)
    Y = _alloc_out(layer, B)
    rs.rsparse_linear(layer, Xd.data_ptr(), B, Y.data_ptr(), stream_ptr())
    out = {"Y": _read_out(layer, Y)}
    if lists:
        out["act"] = [rs.rsparse_last_active(layer, b) for b in range(B)]
        out["union"] = rs.rsparse_last_active(layer, -1)
    return out


def run_dense(layer, X16):
    X16 = np.atleast_2d(X16)
    B = X16.shape[0]
    Xd = to_dev16(X16)
    Y = _alloc_out(layer, B)
    rs.rsparse_dense_ref(layer, Xd.data_ptr(), B, Y.data_ptr(), stream_ptr())
    return _read_out(layer, Y)


def oracle_linear(L, X16, tau, **kw):
    r = L.rank
    return oracle.rsparse_linear(L.W16, L.U16 if r else None, L.SV16 if r else None, np.atleast_2d(X16),
                                 L.dtype, L.dtype, tau, nthreads=8, **kw)


def check_outputs(got, want, out_dtype, rows=None):
    """got / want: [B, d_out] float64.  Per token: relative L2 and max-abs against ||y||_inf."""
    finite = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), finite), "non-finite pattern differs"
    for b in range(want.shape[0]):
        w, g = want[b][finite[b]], got[b][finite[b]]
        if w.size == 0:
            continue
        nrm = np.linalg.norm(w)
        err = np.linalg.norm(g - w)
        if out_dtype == rs.F32:
            assert err <= REL_L2_F32 * nrm + 1e-30, f"token {b}: rel L2 {err / max(nrm, 1e-300):.3e} (fp32 out)"
        else:
            assert err <= REL_L2_16 * nrm + 1e-30, f"token {b}: rel L2 {err / max(nrm, 1e-300):.3e}"
            assert np.max(np.abs(g - w)) <= MAX_ABS_16 * np.max(np.abs(w)) + 1e-30, f"token {b}: max-abs"


def check_lists(got, want):
    assert len(got["act"]) == len(want["act"])
    for b, (g, w) in enumerate(zip(got["act"], want["act"])):
        assert np.array_equal(g, w), f"token {b}: kept-channel list differs ({len(g)} vs {len(w)})"
    assert np.array_equal(got["union"], want["union"]), "union list differs"


def tokens_for(L, n, kind="dmodel", config=80, linear=0, offset=0):
    src = (synth.DModelInput if kind == "dmodel" else synth.DownInput)(L.d_in, config=config, linear=linear)
    return synth.encode16(src.tokens(n, offset=offset), L.dtype), src


def calibrated_tau(L, src, s, n_calib=64):
    Xc = synth.encode16(src.tokens(n_calib, stream=synth.STREAM_CALIB), L.dtype)
    return oracle.quantile_tau(Xc, L.dtype, s)
