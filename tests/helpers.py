"""Shared by the GPU parity tests: tensor <-> oracle conversions and the error metric."""
from oracle.checks import ORC_DT, TOL, rel_err, to_bits, to_f64, weights_bits  # noqa: F401
