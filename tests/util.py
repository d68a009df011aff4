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


def route_without_site(route: np.ndarray, site: int) -> np.ndarray:
    """The route bytes with `site` taken out of every request's choice (a request left with nothing gets 255)."""
    out = route.copy()
    for b, v in enumerate(route):
        v = int(v)
        if v == site:
            out[b] = 255
        elif v != 255 and (v & 0x80) and (v >> site) & 1:
            rest = (v & 0x7F) & ~(1 << site)
            out[b] = (0x80 | rest) if rest else 255
    return out


def lora_visibility(run_oracle, route: np.ndarray, ref_outputs) -> float:
    """How far the outputs move when the LoRA term of one site is dropped, at worst: for every site some
    request uses, the oracle runs again without that site's term, and every request that used it must see
    its outputs change; returns the smallest such change, as the row metric of the tolerances
    (max_j |difference| / max_j |reference|, the larger of the outputs counts).  A parity tolerance far below
    this number cannot be met by a kernel that loses a term."""
    worst = np.inf
    for site in range(7):
        rows = np.array([b for b, v in enumerate(route) if oracle.route_has(int(v), site)], dtype=np.int64)
        if rows.size == 0:
            continue
        dropped = run_oracle(route_without_site(route, site))
        moved = np.zeros(rows.size)
        for full, part in zip(ref_outputs, dropped):
            moved = np.maximum(moved, row_rel_err(part[rows], full[rows]))
        worst = min(worst, float(moved.min()))
    return worst
