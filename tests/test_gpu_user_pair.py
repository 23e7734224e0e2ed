"""A type and an operator compiled OUTSIDE the library (paper Sec. IV-A: any struct of plain fields, any
associative operator the caller writes), handed to ks_scan_pair / ks_mapreduce_pair through the C ABI.
The pairs are those of paper_2603_18695_amd/examples/user_pair.hip, built in-tree by build.py.

References: the 24-byte statistics struct against numpy's own accumulate routines; the affine maps over
Z/2^32 (8 bytes, not commutative) against the definition folded in Python for small inputs, and for
large ones by induction: out[0] = in[0] and every out[i] is out[i-1] followed by in[i], checked at all i."""
import ctypes
import os
import sys

import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

STATS = np.dtype([("sum", "<i8"), ("lo", "<i4"), ("hi", "<i4"), ("cnt", "<u8")])
M32 = (1 << 32) - 1


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ks():
    import paper_2603_18695_amd as ks
    return ks


@pytest.fixture(scope="module")
def pairs(ks):
    lib = ctypes.CDLL(os.path.join(os.path.dirname(ks.LIB_PATH), "examples", "libks_user_pair.so"))
    out = {}
    for name in ("affine_u32", "stats24"):
        fn = getattr(lib, f"ks_user_{name}_pair")
        fn.restype = ctypes.c_void_p
        out[name] = fn()
    assert ks.ks_pair_elem_bytes(out["affine_u32"]) == 8 and ks.ks_pair_elem_bytes(out["stats24"]) == 24
    return out


def words(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x).view(np.int32).reshape(len(x), -1)).cuda()


def random_affine(n, seed):
    return np.random.default_rng(seed).integers(0, 1 << 32, size=(n, 2), dtype=np.uint32)


def compose(e, l):      # first e, then l, over Z/2^32: plain Python integers
    return ((l[0] * e[0]) & M32, (l[0] * e[1] + l[1]) & M32)


def check_affine_scan(x, got, inclusive, what):
    n = len(x)
    if n == 0:
        return
    xa, xb = x[:, 0].astype(np.uint64), x[:, 1].astype(np.uint64)
    ga, gb = got[:, 0].astype(np.uint64), got[:, 1].astype(np.uint64)
    if n <= 30_000:     # the definition itself
        ref = oracle.fold_scan(compose, [(int(a), int(b)) for a, b in x], inclusive, identity=(1, 0))
        assert [(int(a), int(b)) for a, b in got] == ref, what
        return
    if inclusive:       # out[0] = in[0]; out[i] = in[i] after out[i-1]
        assert (int(ga[0]), int(gb[0])) == (int(xa[0]), int(xb[0])), what
        assert np.array_equal(ga[1:], (xa[1:] * ga[:-1]) & M32), what
        assert np.array_equal(gb[1:], (xa[1:] * gb[:-1] + xb[1:]) & M32), what
    else:               # out[0] = identity; out[i] = in[i-1] after out[i-1]
        assert (int(ga[0]), int(gb[0])) == (1, 0), what
        assert np.array_equal(ga[1:], (xa[:-1] * ga[:-1]) & M32), what
        assert np.array_equal(gb[1:], (xa[:-1] * gb[:-1] + xb[:-1]) & M32), what


def test_affine_maps_over_z32(ks, pairs):
    pair = pairs["affine_u32"]
    tile = 15 * 64 * 9 * 2      # elements of the largest tile an 8-byte element can get
    for n in (1, 2, 63, 65, 4097, 30_000, tile - 1, tile + 1, 70 * tile + 5, 700 * tile + 3):
        x = random_affine(n, seed=n % 97)
        d_in = words(x)
        for inclusive in (True, False):
            say(f"[case] user pair affine_u32 n={n} inclusive={inclusive}")
            d_out = torch.zeros_like(d_in)
            ks.ks_scan_pair(pair, d_in, d_out, inclusive=inclusive)
            ks.ks_scan_check()
            check_affine_scan(x, d_out.cpu().numpy().view(np.uint32), inclusive, f"affine_u32 n={n} incl={inclusive}")
        # the reduction is the last element of the inclusive scan (d_out holds the exclusive one now)
        ks.ks_scan_pair(pair, d_in, d_out, inclusive=True)
        one = torch.zeros_like(d_in[:1])
        ks.ks_mapreduce_pair(pair, d_in, one)
        ks.ks_scan_check()
        assert torch.equal(one[0], d_out[-1]), f"reduction n={n}"
    # in place
    x = random_affine(3 * tile + 7, seed=5)
    d = words(x)
    ks.ks_scan_pair(pair, d, d)
    ks.ks_scan_check()
    check_affine_scan(x, d.cpu().numpy().view(np.uint32), True, "in place")


def random_stats(n, seed):
    rng = np.random.default_rng(seed)
    x = np.empty(n, STATS)
    v = rng.integers(-2 ** 31, 2 ** 31, size=n, dtype=np.int64)
    x["sum"] = v * rng.integers(1, 1 << 31, size=n, dtype=np.int64)      # large: the running sum wraps
    x["lo"] = v
    x["hi"] = v
    x["cnt"] = rng.integers(0, 1 << 62, size=n, dtype=np.uint64)
    return x


def stats_reference(x, inclusive):
    with np.errstate(over="ignore"):
        ref = np.empty(len(x), STATS)
        ref["sum"] = np.cumsum(x["sum"].view(np.uint64), dtype=np.uint64).view(np.int64)
        ref["lo"] = np.minimum.accumulate(x["lo"])
        ref["hi"] = np.maximum.accumulate(x["hi"])
        ref["cnt"] = np.cumsum(x["cnt"], dtype=np.uint64)
    if inclusive:
        return ref
    out = np.empty_like(ref)
    out[0] = (0, np.iinfo(np.int32).max, np.iinfo(np.int32).min, 0)
    out[1:] = ref[:-1]
    return out


def test_statistics_struct_of_24_bytes(ks, pairs):
    pair = pairs["stats24"]
    tile = 15 * 64 * 6          # 9 granules per lane hold 6 elements of 24 bytes
    for n in (1, 5, 6, 7, 383, 385, tile - 1, tile, tile + 1, 64 * tile + 1, 700 * tile + 11):
        x = random_stats(n, seed=n % 89)
        d_in = words(x)
        for inclusive in (True, False):
            say(f"[case] user pair stats24 n={n} inclusive={inclusive}")
            d_out = torch.zeros_like(d_in)
            ks.ks_scan_pair(pair, d_in, d_out, inclusive=inclusive)
            ks.ks_scan_check()
            got = d_out.cpu().numpy().reshape(-1).view(STATS)
            assert got.tobytes() == stats_reference(x, inclusive).tobytes(), f"stats24 n={n} incl={inclusive}"
        one = torch.zeros_like(d_in[:1])
        ks.ks_mapreduce_pair(pair, d_in, one)
        ks.ks_scan_check()
        assert one.cpu().numpy().reshape(-1).view(STATS)[0] == stats_reference(x, True)[-1], f"reduction n={n}"
    # an empty reduction writes the operator's identity
    one = torch.zeros((1, 6), dtype=torch.int32, device="cuda")
    ks.ks_mapreduce_pair(pair, torch.zeros((0, 6), dtype=torch.int32, device="cuda"), one)
    ks.ks_scan_check()
    ident = one.cpu().numpy().reshape(-1).view(STATS)[0]
    assert (int(ident["sum"]), int(ident["lo"]), int(ident["hi"]), int(ident["cnt"])) == (0, 2 ** 31 - 1, -2 ** 31, 0)


def test_what_is_not_a_pair_is_refused(ks, pairs):
    lib = ks.raw_library()
    junk = ctypes.create_string_buffer(256)
    p = ctypes.addressof(junk)
    assert ks.ks_pair_elem_bytes(p) == 0
    assert lib.ks_scan_pair(p, 1, 0x10000000, 0x20000000, 16, None) == ks.KS_ERR_INVALID_ARG
    assert lib.ks_mapreduce_pair(None, 0x10000000, 16, 0x20000000, None) == ks.KS_ERR_INVALID_ARG
    good = pairs["stats24"]
    assert lib.ks_scan_pair(good, 1, None, None, 0, None) == ks.KS_OK
    assert lib.ks_scan_pair(good, 1, 0x10000004, 0x20000000, 16, None) == ks.KS_ERR_MISALIGNED     # int64 fields
    assert lib.ks_scan_pair(good, 1, 0x10000000, 0x10000018, 16, None) == ks.KS_ERR_OVERLAP


def test_the_c_abi_from_a_program_without_python(ks):
    # examples/scan_from_c.cpp: hipMalloc, ks_scan, ks_mapreduce, ks_scan_check, ks_release_scratch, its own check
    import subprocess
    exe = os.path.join(os.path.dirname(ks.LIB_PATH), "examples", "scan_from_c")
    say("[case] examples/scan_from_c 5000003")
    r = subprocess.run([exe, "5000003"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "match the host" in r.stdout, r.stdout
