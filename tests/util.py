"""Shared helpers of the parity tests: tolerances, oracle/GPU input bridging, error metrics."""
import numpy as np
import torch

import oracle
from paper_2410_18035_amd import synth

# Output tolerances: relative error per output row, max_j |y - y_ref| / max_j |y_ref|.
TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-5}
# Route parity leaves out prompts whose oracle top-2 logit gap is below margin * std(oracle logits):
# the GPU accumulates in fp32, the oracle in fp64, and a gap of that size can flip on rounding alone.
ROUTE_MARGIN = {torch.bfloat16: 1e-3, torch.float32: 1e-5}


def oracle_adapters(ad: synth.LayerAdapters) -> oracle.Adapters:
    A, B, rank = synth.adapters_as_numpy(ad)
    return oracle.Adapters(A, B, rank)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def row_rel_err(y: np.ndarray, ref: np.ndarray) -> np.ndarray:
    denom = np.abs(ref).max(axis=1)
    denom = np.where(denom == 0, 1.0, denom)
    return np.abs(y - ref).max(axis=1) / denom


def assert_rows_close(y_gpu: torch.Tensor, ref: np.ndarray, dtype, what=""):
    err = row_rel_err(to_f64(y_gpu), ref)
    assert np.isfinite(err).all(), f"{what}: non-finite output"
    assert err.max() <= TOL[dtype], f"{what}: max row rel err {err.max():.3e} > {TOL[dtype]:.0e} (row {err.argmax()})"
    return float(err.max())


def assert_routes_match(route_gpu: torch.Tensor, res: "oracle.RouteResult", dtype, what=""):
    """Bit-exact routes wherever the oracle's decision is not a near-tie; returns the excluded fraction."""
    sigma = float(res.logits.std())
    keep = res.gap >= ROUTE_MARGIN[dtype] * sigma
    got = route_gpu.cpu().numpy()
    bad = np.nonzero(keep & (got != res.route))[0]
    assert bad.size == 0, f"{what}: routes differ at requests {bad.tolist()} (gaps {res.gap[bad]}, sigma {sigma:.3g})"
    return 1.0 - keep.mean()
