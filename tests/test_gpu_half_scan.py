"""Scans of 16-bit floats (bfloat16, IEEE binary16 as bit patterns): every element promoted to float32
as it is loaded, accumulated in float32 (sums: double above one wave's run), every output rounded to
the 16-bit type.  Reference: the oracle's float64 scan of the promoted inputs.  A sum output must
lie within half a unit in the last place of the 16-bit type around the reference, plus the float bar
of the float32 accumulation; running minima and maxima are elements of the input and compare exactly.
Arrays of odd length end in the middle of a dword: what lies behind them must stay untouched."""
import sys

import numpy as np
import pytest
import torch

import ks_inputs
import oracle
from parity import float_bound

pytestmark = pytest.mark.gpu
MANTISSA = {"bf16": 7, "f16": 10}
MIN_EXP = {"bf16": -126, "f16": -14}
SENTINEL = 0x7B7B


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def half_ulp(kind, ref):
    e = np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** MIN_EXP[kind])))
    return 0.5 * 2.0 ** (e - MANTISSA[kind])


def run_scan(ks, kind, op, x, inclusive, how, pad=5):
    """Scan x; the output buffer has `pad` sentinel elements behind it, which must survive."""
    n = len(x)
    d_in = torch.from_numpy(np.concatenate([x, np.full(pad, 0x3C00, np.uint16)]).view(np.int16)).cuda()
    d_out = torch.full((n + pad,), SENTINEL, dtype=torch.int16, device="cuda")
    if how == "in_place":
        d_out[:n] = d_in[:n]
        ks.ks_scan(d_out[:n], d_out[:n], dtype=kind, op=op, inclusive=inclusive)
    elif how == "plain":
        ks.ks_scan(d_in[:n], d_out[:n], dtype=kind, op=op, inclusive=inclusive)
    else:
        temp = torch.empty(ks.ks_scan_temp_bytes(dtype=kind, op=op, n=n, algo=how), dtype=torch.uint8, device="cuda")
        ks.ks_scan_with_temp(d_in[:n], d_out[:n], temp, dtype=kind, op=op, inclusive=inclusive, algo=how)
    ks.ks_scan_check()
    out = d_out.cpu().numpy().view(np.uint16)
    assert np.all(out[n:] == SENTINEL), f"wrote behind the output ({kind},{op}) n={n} {how}"
    return out[:n]


def check(kind, op, x, got_bits, inclusive, what):
    vals = oracle.apply_map("widen_f32", x, kind)
    got = oracle.apply_map("widen_f32", got_bits, kind).astype(np.float64)
    ref = oracle.scan(op, "f32", vals, inclusive).astype(np.float64)
    if op == "sum":
        bound = half_ulp(kind, ref) + float_bound(ref)
        bad = np.abs(got - ref) > bound
        assert not bad.any(), f"{what}: {int(bad.sum())} outputs off, first at {int(np.argmax(bad))}: " \
                              f"{got[np.argmax(bad)]} vs {ref[np.argmax(bad)]}"
    else:
        assert np.array_equal(got, ref), what


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("op", ["sum", "max", "min"])
def test_edge_sizes_both_strategies(ks, kind, op):
    small, big = 3 * 64 * 8 * 8, 15 * 64 * 8 * 8         # tiles of the 4 x 8 and the 16 x 8 shape, in elements
    sizes = [1, 2, 3, 7, 8, 9, 511, 512, 513, small - 1, small, small + 1, 64 * small + 3, big + 1, 5 * small * 64 + 7,
             70 * big + 5, 300 * big + 2, 700 * big + 3]
    for n in sizes:
        # sums: values in (-1, 1), what the absolute part of the float bar is derived for
        x = ks_inputs.random_half_bits(kind, n, seed=n % 97, spikes=(op != "sum"))
        for inclusive in (True, False):
            for how in ("plain", "reduce_then_scan", "lookback") if n < 2_000_000 else ("plain",):
                say(f"[case] ({kind},{op}) n={n} inclusive={inclusive} {how}")
                check(kind, op, x, run_scan(ks, kind, op, x, inclusive, how), inclusive, f"({kind},{op}) n={n} {how}")
        say(f"[case] ({kind},{op}) n={n} in place")
        check(kind, op, x, run_scan(ks, kind, op, x, True, "in_place"), True, f"({kind},{op}) n={n} in place")


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_closed_forms_and_rules(ks, kind):
    one = {"bf16": 0x3F80, "f16": 0x3C00}[kind]
    n = 2 ** (MANTISSA[kind] + 1) - 1      # 1, 2, 3, ...: every count up to 2^(p+1) is a value of the format
    got = run_scan(ks, kind, "sum", np.full(n, one, np.uint16), True, "plain")
    assert np.array_equal(oracle.apply_map("widen_f32", got, kind), np.arange(1, n + 1, dtype=np.float32))
    # beyond the format's integers the outputs are the counts rounded to nearest, ties to even
    n = 300_001 if kind == "bf16" else 60_001
    got = oracle.apply_map("widen_f32", run_scan(ks, kind, "sum", np.full(n, one, np.uint16), True, "plain"), kind)
    counts = np.arange(1, n + 1, dtype=np.float64)
    assert np.all(np.abs(got - counts) <= half_ulp(kind, counts))
    # both arrays start on a dword; anything else is refused, and so are strided views
    x = torch.zeros(128, dtype=torch.int16, device="cuda")
    with pytest.raises(ks.KsError) as e:
        ks.ks_scan(x[1:33], x[65:97], dtype=kind, op="sum")
    assert e.value.status == ks.KS_ERR_MISALIGNED
    with pytest.raises(ks.KsError) as e:
        ks.ks_scan_strided(x, x.clone(), dtype=kind, op="sum", n=8, in_stride=2, out_stride=2)
    assert e.value.status == ks.KS_ERR_UNSUPPORTED


def test_large_bf16_cumsum(ks):
    n = (1 << 28) + 1                  # 512 MiB each way, odd length
    x = ks_inputs.random_half_bits("bf16", 1 << 20, seed=7, spikes=False)
    x = np.tile(x, (n >> 20) + 1)[:n]
    say(f"[case] (bf16,sum) n={n}")
    check("bf16", "sum", x, run_scan(ks, "bf16", "sum", x, True, "plain"), True, f"(bf16,sum) n={n}")
