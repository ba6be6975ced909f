"""Helpers shared by the tests: tensor -> float64 arrays, the float tolerance."""
import numpy as np
import torch


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 / fp32) tensor to a float64 NumPy array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def i64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").numpy()


# Float bar of the build: max-abs-err <= 2e-2 relative to output RMS for bf16 with
# fp32 accumulation, read per token row against the unrounded float64 oracle
# (a row's scale is set by its combine weights, so one global RMS would put the
# bound below the bf16 rounding step of the largest rows).
ROW_TOL = 2e-2


# Float bars for the backward pass, which the benchmark spec does not state.  The library stores
# the derivatives p = dH/da, q = dH/db of the SwiGLU product, the activations H and the gradients
# da = dH p, db = dH q in bf16 (da, db and H are MFMA operands), and the float64 oracle stores
# nothing rounded.  One bf16 rounding perturbs a value by a relative 2^-9 at most, about 1e-3 in
# the root mean square; every gradient term carries two of them (the stored derivative and the
# stored product, or H alone for dW_down), so the error of an output row, taken in the root mean
# square over the row, is about sqrt(2) * 1e-3 .. 3e-3 of the row's RMS whatever the number of
# rows summed (error and value grow alike).  A float64 computation that only rounds those five
# tensors measures 0.0027 .. 0.004 on every shape tried, from one-row groups to thousands of
# rows.  BWD_RMS_TOL is 1e-2.
# The largest single error of a row is heavy-tailed instead: da is a product of three random
# factors, and a one-row group has no sum to average over, so that same computation reaches
# 0.01 .. 0.035 of the row RMS.  BWD_MAX_TOL = 8e-2 (four times the forward bar) only guards
# against isolated wrong elements; the RMS bar is the one that carries the parity claim.
BWD_RMS_TOL = 1e-2
BWD_MAX_TOL = 8e-2


def row_rms_err(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    """rms_i(got - want) / rms_i(want) per row; all-zero oracle rows must match exactly."""
    err = np.sqrt(((got - want) ** 2).mean(axis=1))
    rms = np.sqrt((want ** 2).mean(axis=1))
    out = np.zeros_like(err)
    nz = rms > 0
    out[nz] = err[nz] / rms[nz]
    out[~nz] = np.where(err[~nz] == 0, 0.0, np.inf)
    return out


def row_rel_err(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    """max_i |got - want| / rms_i(want) per row; rows whose oracle value is all
    zero must match exactly (reported as 0 or inf)."""
    err = np.abs(got - want).max(axis=1)
    rms = np.sqrt((want ** 2).mean(axis=1))
    out = np.zeros_like(err)
    nz = rms > 0
    out[nz] = err[nz] / rms[nz]
    out[~nz] = np.where(err[~nz] == 0, 0.0, np.inf)
    return out


def bf16_rounding_excess(got: np.ndarray, want: np.ndarray) -> float:
    """For an INTERMEDIATE kept in bf16 (the SwiGLU activations H): every element
    must sit within one bf16 rounding step of the oracle value, plus a small
    allowance (1e-3 of the row RMS) for fp32 accumulation order and the fast
    exponential.  H rows are heavy-tailed (a product of two near-Gaussians), so
    their largest element's rounding step alone can exceed 2e-2 of the row RMS;
    the 2e-2 bar applies to the layer's outputs, not to this intermediate.
    Returns max over elements of |err| / allowed (<= 1 passes)."""
    rms = np.sqrt((want ** 2).mean(axis=1, keepdims=True))
    allowed = 2.0 ** -8 * np.abs(want) + 1e-3 * rms + 1e-30
    return float((np.abs(got - want) / allowed).max())
