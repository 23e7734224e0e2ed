"""ks_scan_seeded: out[i] = seed op in[0] op ... op in[i], one piece of a longer sequence.  Reference:
the oracle's plain scan of the sequence with the seed put in front (the definition: the seed is one
more element on the left), and the whole-array scan that a chain of seeded pieces has to reproduce."""
import sys

import numpy as np
import pytest
import torch

import ks_inputs
import oracle
from parity import KINDS, assert_matches, random_input, reference, to_device, to_host

pytestmark = pytest.mark.gpu

PAIRS = [("i32", "sum"), ("f32", "sum"), ("u64", "max"), ("f64", "min"), ("affine_f32", "affine_compose"),
         ("argmax_i32_cnt64", "argmax_count"), ("mat2_u32", "mat2_mul"), ("quat_f32", "quat_mul"),
         ("mat2_u64", "mat2_mul"), ("range_i32_cnt32", "range_count")]


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("dtype,op", PAIRS)
def test_seed_in_front_of_the_sequence(ks, dtype, op):
    eb = ks.ks_elem_bytes(dtype)
    big = 15 * 64 * 9 * 16 // eb
    for n in (1, 2, 65, 3 * 64 * 8 * 16 // eb + 1, big - 1, big + 1, 64 * big + 3, 300 * big + 7):
        x = random_input(dtype, op, n + 1, seed=n % 83 + 1)       # x[0] plays the seed
        d_all = to_device(x)
        d_seed, d_in = d_all[:1], d_all[1:]
        for inclusive in (True, False):
            say(f"[case] seeded ({dtype},{op}) n={n} inclusive={inclusive}")
            d_out = torch.zeros_like(d_in)
            ks.ks_scan_seeded(d_in, d_out, d_seed, dtype=dtype, op=op, inclusive=inclusive)
            ks.ks_scan_check()
            # the definition: scan the sequence with the seed in front, drop the seed's own position
            ref = reference(dtype, op, x, inclusive)[1:] if inclusive else reference(dtype, op, x, False)[1:]
            assert_matches(dtype, op, to_host(d_out, x.dtype), ref, f"seeded ({dtype},{op}) n={n} incl={inclusive}")


@pytest.mark.parametrize("dtype,op", [("i32", "sum"), ("mat2_u32", "mat2_mul"), ("argmax_i32_cnt64", "argmax_count"),
                                      ("mat2_u64", "mat2_mul")])
def test_pieces_chained_by_their_seeds_give_the_whole_scan(ks, dtype, op):
    # an array scanned in four pieces of different sizes, every piece seeded with the last output of the
    # piece before it (read from the output array on the device, no host round trip): bit for bit the
    # scan of the whole array.  This is the single-device form of scanning shard by shard.
    n = 5_000_011
    x = random_input(dtype, op, n, seed=17)
    d_in = to_device(x)
    d_out = torch.zeros_like(d_in)
    cuts = [0, 1, 700_001, 700_002 + 2_345_678, n]
    say(f"[case] chained pieces ({dtype},{op}) n={n} cuts={cuts}")
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        if lo == 0:
            ks.ks_scan(d_in[lo:hi], d_out[lo:hi], dtype=dtype, op=op)
        else:
            ks.ks_scan_seeded(d_in[lo:hi], d_out[lo:hi], d_out[lo - 1:lo], dtype=dtype, op=op)
    ks.ks_scan_check()
    assert_matches(dtype, op, to_host(d_out, x.dtype), reference(dtype, op, x, True), f"chained ({dtype},{op})")


def test_seeded_sixteen_bit_floats_and_argument_checks(ks):
    n = 400_001
    x = ks_inputs.random_half_bits("bf16", n + 2, seed=3, spikes=False)
    d = torch.from_numpy(x.view(np.int16)).cuda()
    out = torch.zeros(n, dtype=torch.int16, device="cuda")
    ks.ks_scan_seeded(d[2:], out, d[1:2], dtype="bf16", op="sum")        # the seed itself may sit at any 2-byte address
    ks.ks_scan_check()
    vals = oracle.apply_map("widen_f32", x[1:], "bf16")
    ref = oracle.scan("sum", "f32", vals, True)[1:].astype(np.float64)
    got = oracle.apply_map("widen_f32", out.cpu().numpy().view(np.uint16), "bf16").astype(np.float64)
    half_ulp = 0.5 * 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126))) - 7)
    assert np.all(np.abs(got - ref) <= half_ulp + np.maximum(1e-4 * np.abs(ref), 1e-3))
    lib = ks.raw_library()
    assert lib.ks_scan_seeded(0, 0, 1, 0x10000000, 0x20000000, 16, None, None) == ks.KS_ERR_INVALID_ARG    # no seed
    assert lib.ks_scan_seeded(0, 0, 1, 0x10000000, 0x20000000, 16, 0x30000002, None) == ks.KS_ERR_MISALIGNED
    assert lib.ks_scan_seeded(0, 0, 1, None, None, 0, None, None) == ks.KS_OK                               # n == 0
