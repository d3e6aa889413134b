"""Checker-side conversions and the error metric (test infrastructure, like the rest of oracle/):
tensor <-> the arrays the oracle takes, and the tolerance the parity tests, the smoke test and the
bench's CPU leg compare with.  Nothing here is on the product path."""
import numpy as np
import torch

ORC_DT = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}
# relative tolerance of layer outputs against the fp64 oracle, per activation type
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2, torch.float16: 2e-2}

# Gradients of a layer with 2-byte activations against the fp64 oracle fed the unrounded incoming
# gradient: the device rounds the masked gradient to the activation type before the two matrix
# products (relative error up to 2^-9 per element for bf16, 2^-11 for fp16, independent from element
# to element; a sum of n products carries about 2^-9 / sqrt(3) of the root sum of squares of its
# terms, the largest of some 10^5 outputs about 5 times that, and rel_err's rms floor adds the spread
# of the rows' magnitudes, e.g. the 1/terms scaling of a normalised aggregate: about 2.5e-2 observed
# for bf16 at 256 output columns, reproduced on the CPU by feeding the oracle the rounded gradient).
# The sharp comparison is against the oracle fed the gradient rounded the same way: GRAD_TOL_SAME.
GRAD_TOL = {torch.float32: 2e-5, torch.bfloat16: 4e-2, torch.float16: 5e-3}
GRAD_TOL_SAME = 3e-5


def round_like(x: np.ndarray, dt) -> np.ndarray:
    """x rounded to dt (round to nearest even) and widened to float64: the incoming gradient as a
    2-byte layer's matrix products take it."""
    if dt == torch.float32:
        return np.asarray(x, np.float64)
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(dt).to(torch.float64).numpy()


def chain_tol(dt, n_layers: int) -> float:
    """Bound for the last rows of a whole chain of layers against the oracle's own chain.
    fp32: the layer bound itself (stored activations are the fp32 results; the per-layer error of
    about 1e-6 adds up to well under 1e-5 over the depths used).  2-byte types: both sides round
    every layer's activations to the storage type, and where the two fp32 results straddle a
    rounding boundary the stored values differ by one unit in the last place (2^-8 relative for
    bf16), which the next layer carries on: one layer bound per layer.  Isolated layers (the same
    stored inputs on both sides) always meet TOL."""
    return TOL[dt] if dt == torch.float32 else TOL[dt] * n_layers


def to_bits(t: torch.Tensor) -> np.ndarray:
    """Host numpy array the oracle understands (uint16 bit patterns for 2-byte floats)."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def rel_err(got64: np.ndarray, ref64: np.ndarray) -> float:
    """max |got - ref| / max(|ref|, rms(ref)): element-wise relative error with
    the tensor's rms as the floor (plain relative error is undefined at ReLU zeros)."""
    if ref64.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref64 ** 2)))
    den = np.maximum(np.abs(ref64), max(rms, 1e-30))
    return float(np.max(np.abs(got64 - ref64) / den))


def weights_bits(weights):
    return [(to_bits(a), to_bits(b), None if c is None else to_bits(c)) for a, b, c in weights]
