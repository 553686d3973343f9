"""Seeded synthetic inputs for the R-Sparse linear layer: weights, factors, tokens.

This module only *generates* operands.  It holds none of the method's
arithmetic (no thresholding, no index lists, no sparse or low-rank products,
no quantile): both the CPU oracle's tests and the HIP path's tests draw their
inputs from here, and neither implementation lives here.  numpy only.

Recipe (stand-in for real Llama weights/activations, which are not available):

* W = U diag(sigma) V^T with U [d_out, p], V [d_in, p] the sign-fixed thin-QR
  factors of seeded N(0,1) matrices, p = min(d_in, d_out) and
  sigma_i = 0.5 * i^-0.6.  The singular factors of W are therefore known in
  closed form (Sec. 3.3 writes the layer through exactly this decomposition).
  W is rounded once to the 16-bit storage type.
* The rank-r factors handed to the library are U_r = U[:, :r] and
  S_r V_r^T = diag(sigma[:r]) V[:, :r]^T (Sec. 3.4 splits Sigma evenly between
  the two sides; folding all of it into the V side gives the same product and
  keeps U_r's entries well scaled in 16 bits), each rounded once.
* Inputs of d_model-wide linears: x_c = s_c * Laplace(0,1), with a fixed
  per-channel scale s_c ~ LogNormal(0, 0.5) and 8 outlier channels scaled x20:
  heavy-tailed with a few dominant channels, which is the structure the method
  exploits (Sec. 1, Fig. 1).
* Inputs of the MLP down projection: SiLU(g) * u with g, u ~ N(0,1)
  (Sec. 3.1, H = X W_up^T (.) sigma(X W_gate^T)).

Every stream has its own seed: 1000*config + 10*linear + stream, with stream
0: U, 1: V, 2: channel scales and outlier picks, 3: calibration tokens,
4: timed / tested tokens.
"""
from __future__ import annotations

import numpy as np

F16 = 0
BF16 = 1
DTYPE_NAMES = {F16: "f16", BF16: "bf16"}

STREAM_U, STREAM_V, STREAM_SCALES, STREAM_CALIB, STREAM_TOKENS = range(5)


def seed_for(config: int, linear: int, stream: int) -> int:
    return 1000 * config + 10 * linear + stream


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------------------
# 16-bit storage encodings (format conversions only)
# ---------------------------------------------------------------------------

def encode16(a, dtype: int) -> np.ndarray:
    """Round a float array once (nearest-even) to fp16 / bf16; return the uint16 bits."""
    a = np.asarray(a)
    if dtype == F16:
        with np.errstate(over="ignore"):
            return np.ascontiguousarray(a.astype(np.float16)).view(np.uint16)
    if dtype == BF16:
        with np.errstate(over="ignore"):
            f = np.ascontiguousarray(a.astype(np.float32))
        u = f.view(np.uint32).astype(np.uint64)
        nan = np.isnan(f)
        if a.dtype == np.float64:
            # one rounding from fp64: if the fp32 step landed exactly on a bf16 tie that `a` was not on, move one
            # fp32 step towards `a` so that the second rounding falls on a's side
            with np.errstate(invalid="ignore"):
                fd = f.astype(np.float64)
                tie = ((u & 0xFFFF) == 0x8000) & np.isfinite(f) & (fd != a)
                up = np.abs(a) > np.abs(fd)
            u = np.where(tie & up, u + 1, np.where(tie & ~up, u - 1, u))
        rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
        out = rounded.astype(np.uint16)
        out[nan] = 0x7FC0
        return out
    raise ValueError("dtype must be F16 or BF16")


def decode16(bits, dtype: int) -> np.ndarray:
    """Exact widening of fp16 / bf16 bits to float64."""
    bits = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16))
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError("dtype must be F16 or BF16")


# ---------------------------------------------------------------------------
# weights and factors
# ---------------------------------------------------------------------------

def orthonormal(seed: int, n: int, p: int) -> np.ndarray:
    """[n, p] matrix with orthonormal columns: thin-QR Q of a seeded N(0,1) matrix,
    column signs fixed so that diag(R) > 0 (makes the factor unique)."""
    a = _rng(seed).standard_normal((n, p))
    q, r = np.linalg.qr(a, mode="reduced")
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return q * s


def spectrum(p: int, scale: float = 0.5, decay: float = 0.6) -> np.ndarray:
    return scale * np.arange(1, p + 1, dtype=np.float64) ** (-decay)


class Layer:
    """One synthetic linear layer and its rank-r factors (float64 and stored 16-bit)."""

    def __init__(self, d_in, d_out, rank, dtype, U, sigma, V):
        self.d_in, self.d_out, self.rank, self.dtype = d_in, d_out, rank, dtype
        self.U, self.sigma, self.V = U, sigma, V           # float64, closed form
        W = (U * sigma) @ V.T                              # [d_out, d_in] float64
        self.W16 = encode16(W, dtype)                      # stored weight bits
        self.U16 = encode16(U[:, :rank], dtype)            # [d_out, r]
        self.SV16 = encode16((V[:, :rank] * sigma[:rank]).T, dtype)   # [r, d_in]

    def permuted_channels(self, perm) -> "Layer":
        """The layer W[:, perm]: same U and sigma, V's rows permuted.  Still an exact
        U diag(sigma) V'^T with orthonormal V'; used to fill a ring of distinct layers
        cheaply (distinct HBM addresses, same construction)."""
        perm = np.asarray(perm)
        out = object.__new__(Layer)
        out.d_in, out.d_out, out.rank, out.dtype = self.d_in, self.d_out, self.rank, self.dtype
        out.U, out.sigma = self.U, self.sigma
        out.V = None if self.V is None else self.V[perm]
        out.W16 = np.ascontiguousarray(self.W16[:, perm])
        out.U16 = self.U16
        out.SV16 = np.ascontiguousarray(self.SV16[:, perm])
        return out


def make_layer(d_in: int, d_out: int, rank: int, dtype: int, config: int = 0,
               linear: int = 0, sigma=None) -> Layer:
    p = min(d_in, d_out)
    if not 0 <= rank <= p:
        raise ValueError("rank must be in [0, min(d_in, d_out)]")
    U = orthonormal(seed_for(config, linear, STREAM_U), d_out, p)
    V = orthonormal(seed_for(config, linear, STREAM_V), d_in, p)
    sig = spectrum(p) if sigma is None else np.asarray(sigma, dtype=np.float64)
    return Layer(d_in, d_out, rank, dtype, U, sig, V)


# ---------------------------------------------------------------------------
# activations
# ---------------------------------------------------------------------------

class DModelInput:
    """Heavy-tailed d_model-wide activations with a few outlier channels."""

    def __init__(self, d: int, config: int = 0, linear: int = 0, n_outliers: int = 8,
                 outlier_scale: float = 20.0):
        g = _rng(seed_for(config, linear, STREAM_SCALES))
        self.d = d
        self.scale = np.exp(0.5 * g.standard_normal(d))
        self.outliers = np.sort(g.choice(d, size=min(n_outliers, d), replace=False))
        self.scale[self.outliers] *= outlier_scale
        self.config, self.linear = config, linear

    def tokens(self, n: int, stream: int = STREAM_TOKENS, offset: int = 0) -> np.ndarray:
        """[n, d] float64 tokens; `offset` gives disjoint token sets per stream."""
        g = _rng(seed_for(self.config, self.linear, stream) + 100_000 * offset)
        return self.scale * g.laplace(0.0, 1.0, size=(n, self.d))


class DownInput:
    """Input of the MLP down projection: SiLU(g) * u, g and u i.i.d. N(0,1)."""

    def __init__(self, d: int, config: int = 0, linear: int = 0):
        self.d, self.config, self.linear = d, config, linear

    def tokens(self, n: int, stream: int = STREAM_TOKENS, offset: int = 0) -> np.ndarray:
        rng = _rng(seed_for(self.config, self.linear, stream) + 100_000 * offset)
        g = rng.standard_normal((n, self.d))
        u = rng.standard_normal((n, self.d))
        return g / (1.0 + np.exp(-g)) * u


class GateUpPair:
    """The two operands of the gated MLP input (Sec. 3.1), as a decoder would hand them over: g (gate
    branch) and u (up branch), i.i.d. N(0,1), the same draws DownInput multiplies together.  The
    product itself is the method's business and is not formed here."""

    def __init__(self, d: int, config: int = 0, linear: int = 0):
        self.d, self.config, self.linear = d, config, linear

    def tokens(self, n: int, stream: int = STREAM_TOKENS, offset: int = 0):
        rng = _rng(seed_for(self.config, self.linear, stream) + 100_000 * offset)
        g = rng.standard_normal((n, self.d))
        u = rng.standard_normal((n, self.d))
        return g, u


def random_layer(d_in: int, d_out: int, rank: int, dtype: int, seed: int) -> Layer:
    """Cheap stand-in for very large shapes where the QR construction is too slow for a test:
    i.i.d. Gaussian W and factors with the same entry scales as make_layer's (W rms
    ~ sqrt(sum sigma^2 / (d_in d_out)), U entries ~ 1/sqrt(d_out), S V^T entries ~ sigma_i/sqrt(d_in)).
    The factors are NOT the SVD of W -- parity of the kernels against the oracle does not need
    them to be; accuracy statements do, and never use this generator."""
    g = _rng(seed)
    p = min(d_in, d_out)
    sig = spectrum(p)
    out = object.__new__(Layer)
    out.d_in, out.d_out, out.rank, out.dtype = d_in, d_out, rank, dtype
    out.U = out.V = None
    out.sigma = sig
    w_rms = np.sqrt(np.sum(sig ** 2) / (d_in * d_out))
    out.W16 = encode16(g.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(w_rms), dtype)
    out.U16 = encode16(g.standard_normal((d_out, rank), dtype=np.float32) / np.float32(np.sqrt(d_out)), dtype)
    sv = g.standard_normal((rank, d_in), dtype=np.float32) * (sig[:rank, None] / np.sqrt(d_in)).astype(np.float32)
    out.SV16 = encode16(sv, dtype)
    return out


def quantize_q4(W, dtype: int, group: int = 128):
    """Synthetic 4-bit weights in GPTQ's storage format (Sec. 4.4 combines R-Sparse with GPTQ, group
    128): per output row and group of `group` input channels a 16-bit scale and a 4-bit zero point,
    codes in 0..15.  GPTQ itself needs calibration activations; this input generator rounds to nearest
    on the same asymmetric min/max grid, which fills the format with realistic code, scale and
    zero-point statistics.  Returns (Q uint8 [d_out, d_in], S16 bits [d_out, G], Z uint8 [d_out, G]).
    What the codes mean as weights is the method's business and is not computed here."""
    W = np.asarray(W, dtype=np.float64)
    d_out, d_in = W.shape
    if d_in % group:
        raise ValueError("d_in must be a multiple of the group size")
    G = d_in // group
    Wg = W.reshape(d_out, G, group)
    lo = np.minimum(Wg.min(axis=2), 0.0)
    hi = np.maximum(Wg.max(axis=2), 0.0)
    scale = (hi - lo) / 15.0
    scale[scale == 0.0] = 1.0
    S16 = encode16(scale, dtype)
    s = decode16(S16, dtype)                   # the grid is laid on the scale as stored
    s[s == 0.0] = 1.0
    Z = np.clip(np.rint(-lo / s), 0, 15)
    Q = np.clip(np.rint(Wg / s[:, :, None]) + Z[:, :, None], 0, 15)
    return (np.ascontiguousarray(Q.reshape(d_out, d_in).astype(np.uint8)), S16,
            np.ascontiguousarray(Z.astype(np.uint8)))
