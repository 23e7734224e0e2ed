"""Where the floating point bar comes from: a numpy model of the GPU's tiling (CPU only).

The bar for float32 sums is |gpu - ref64| <= max(1e-4 |ref64|, 1e-3).  On mixed-sign input of
amplitude 1 the running sum is a random walk that reaches several thousand and keeps returning to
zero, where only the absolute 1e-3 is left.  What a scan can reach there depends on where it rounds:

  * a plain float32 left fold rounds every partial sum at the magnitude of the walk and ends up
    tens of bars off: an all-float32 scan is not good enough, whatever its order;
  * the library's tiling rounds in float32 only inside one wave's run (2304 neighbouring elements,
    partial sums of a few dozen) and carries everything above a run (wave totals, tile aggregates,
    the chain of tile prefixes) in double.  The error left is the float32 roundings inside the
    runs: about 1e-6 per run total, a random walk over the runs, i.e. about 1e-4 after 10^4 runs.

The model below takes the tile geometry of the default float32 kernel (15 data waves x 64 lanes x
9 rows x 4 elements = 34560 elements per tile, 2304 per wave) and the kernel's order of additions
inside a run: a left fold inside each 4-element granule, a doubling-step scan of the 64 granule
totals of a row (six levels), a left fold over the nine row totals, two more additions per element
to put the pieces together, one to add the prefix.  That is about twenty roundings on the way to a
run total, each at the size of a partial sum of the run; a plain sequential float32 fold of the run
would take 2304 (and that variant of the model is checked to be worse).  It is a model of the
arithmetic only, written in numpy, and shares nothing with the HIP sources.
"""
import numpy as np

import oracle

ROWS, LANES, G = 9, 64, 4
RUN = ROWS * LANES * G    # elements one wave scans in float32
RTOL, ATOL = 1e-4, 1e-3


def worst_ratio(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref) / np.maximum(RTOL * np.abs(ref), ATOL)))


def run_scan_hierarchical(runs):
    """float32 inclusive scan inside each run, additions grouped as granule -> lanes -> rows."""
    f32 = np.float32
    x = runs.reshape(-1, ROWS, LANES, G)                      # element order: row, lane, position in granule
    g = np.cumsum(x, axis=3, dtype=f32)                       # left fold inside the granule
    inc = g[..., G - 1].copy()                                # granule totals, then scanned over the lanes
    d = 1
    while d < LANES:
        shifted = np.zeros_like(inc)
        shifted[..., d:] = inc[..., :-d]
        inc = (shifted + inc).astype(f32)
        d *= 2
    before_lane = np.zeros_like(inc)
    before_lane[..., 1:] = inc[..., :-1]
    row_total = inc[..., LANES - 1]
    carry = np.zeros_like(row_total)                          # rows before row j, left fold
    for j in range(1, ROWS):
        carry[:, j] = (carry[:, j - 1] + row_total[:, j - 1]).astype(f32)
    base = (carry[..., None] + before_lane).astype(f32)
    return (base[..., None] + g).astype(f32).reshape(-1, RUN)


def run_scan_sequential(runs):
    return np.cumsum(runs, axis=1, dtype=np.float32)


def tiled_scan(x, chain_dtype, run_scan=run_scan_hierarchical):
    """Inclusive sum: float32 inside runs of RUN elements, run totals and their prefix chain in chain_dtype."""
    n = len(x)
    pad = (-n) % RUN
    runs = np.concatenate([x, np.zeros(pad, np.float32)]).reshape(-1, RUN)
    local = run_scan(runs)
    totals = local[:, -1].astype(chain_dtype)
    before = np.concatenate([[chain_dtype(0)], np.cumsum(totals, dtype=chain_dtype)[:-1]])   # exclusive chain
    out = before.astype(np.float32)[:, None] + local                      # one float32 add per element
    return out.reshape(-1)[:n]


def test_float32_tiling_with_double_chain_stays_well_inside_the_bar():
    n = 24_000_000
    x = np.random.default_rng(2024).uniform(-1.0, 1.0, size=n).astype(np.float32)
    ref = oracle.scan("sum", "f32", x, True)
    assert np.abs(ref).max() > 1000.0 and np.abs(ref).min() < 0.01      # the walk is large and crosses zero
    modelled = worst_ratio(tiled_scan(x, np.float64), ref)
    print(f"double chain: worst ratio {modelled:.3f}")
    assert modelled < 0.5                                               # typically 0.1-0.2
    # a sequential float32 fold inside the runs (2304 roundings per run total instead of about twenty)
    seq_runs = worst_ratio(tiled_scan(x, np.float64, run_scan_sequential), ref)
    print(f"double chain, sequential runs: worst ratio {seq_runs:.3f}")
    assert seq_runs > modelled
    # the same tiling with the chain in float32 rounds once per run at the magnitude of the walk
    chain32 = worst_ratio(tiled_scan(x, np.float32), ref)
    print(f"float32 chain: worst ratio {chain32:.3f}")
    assert chain32 > 2 * modelled
    # and a plain float32 left fold is far outside
    fold32 = worst_ratio(np.cumsum(x, dtype=np.float32), ref)
    print(f"float32 left fold: worst ratio {fold32:.1f}")
    assert fold32 > 5.0


def test_model_error_grows_slowly_with_the_number_of_runs():
    # the derivation's scaling: the error is a random walk over the runs, so sixteen times the
    # elements give about four times the error near zero; at the largest size the GPU sweep uses
    # (6.25e7 float32 elements) the model is still inside the bar
    rng = np.random.default_rng(7)
    ratios = []
    for n in (4_000_000, 16_000_000, 64_000_000):
        x = rng.uniform(-1.0, 1.0, size=n).astype(np.float32)
        ref = oracle.scan("sum", "f32", x, True)
        ratios.append(worst_ratio(tiled_scan(x, np.float64), ref))
    print("worst ratio at 4e6 / 1.6e7 / 6.4e7:", ratios)
    assert ratios[2] < 0.8
    assert ratios[2] < 16 * ratios[0]


def test_headline_workload_is_bound_by_the_relative_part():
    # values in [0, 1): the sum grows like n / 2, the bar like 1e-4 n / 2, the modelled error stays at
    # a few ulp of the running sum (ulp(2^20) = 0.125 against a bar of 100 at n = 2^21)
    n = 1 << 21
    x = np.random.default_rng(1).random(size=n, dtype=np.float32)
    ref = oracle.scan("sum", "f32", x, True)
    assert worst_ratio(tiled_scan(x, np.float64), ref) < 0.05
