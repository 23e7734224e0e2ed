"""Shape search for the look-back kernel on the GPU at hand.

The paper leaves an automated search over kernel parameters as future work
(Sec. VI, architecture-specific parameters; Sec. VIII).  This is that search for
one architecture: for a (dtype, op) pair and a size it times every compiled
combination of

    waves     4, 8, 16 wave64s per workgroup
    rows      4, 8, 9, 12, 16  16-byte vectors per thread
    prefetch  next tile requested before the look-back wait, or not
    form      0 common loop (4 and 8 waves), 1 separate loops, 2 separate loops + blocked
              arrangement (16 waves)

through the library's own options (ks_set_option) and prints them best first,
next to the library's built-in default.  Combinations that do not fit the
register file or LDS for the element type are refused by the library
(KS_ERR_UNSUPPORTED) and listed as such.

    python -m paper_2603_18695_amd.tune --dtype f32 --op sum --log2n 28
    python -m paper_2603_18695_amd.tune --dtype u64 --op sum --log2n 27 --exclusive
    python -m paper_2603_18695_amd.tune --dtype f32 --op sum --n 10000000

Inputs are zero-initialised device buffers of the requested size unless
--random is given (random bytes are fine for every integer and struct type;
float types then get uniform [0, 1) values).  Timing uses HIP events around
`--steps` launches after `--warmup` launches.
"""
from __future__ import annotations

import argparse
import itertools
import sys

import torch

import paper_2603_18695_amd as ks

WAVES = (4, 8, 16)
ROWS = (4, 8, 9, 12, 16)
FORMS = {4: (0,), 8: (0,), 16: (1, 2)}


def _buffers(dtype: str, n: int, random: bool):
    nbytes = n * ks.ks_elem_bytes(dtype)
    if dtype in ("f32", "affine_f32", "quat_f32") and random:
        d_in = torch.rand(nbytes // 4, dtype=torch.float32, device="cuda")
    elif dtype == "f64" and random:
        d_in = torch.rand(nbytes // 8, dtype=torch.float64, device="cuda")
    elif random:
        d_in = torch.randint(0, 1 << 20, (nbytes // 4,), dtype=torch.int32, device="cuda")
    else:
        d_in = torch.zeros(nbytes // 4, dtype=torch.int32, device="cuda")
    return d_in, torch.empty_like(d_in)


def _time(dtype, op, inclusive, d_in, d_out, steps, warmup) -> float:
    def launch():
        ks.ks_scan(d_in, d_out, dtype=dtype, op=op, inclusive=inclusive)
    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        launch()
    e1.record()
    torch.cuda.synchronize()
    ks.ks_scan_check()
    return e0.elapsed_time(e1) / steps


def search(dtype: str, op: str, n: int, inclusive: bool = True, steps: int = 30, warmup: int = 4,
           random: bool = False, out=sys.stdout):
    """Time every shape; returns [(ms, waves, rows, prefetch, form)] sorted best first."""
    d_in, d_out = _buffers(dtype, n, random)
    nbytes = 2 * n * ks.ks_elem_bytes(dtype)
    results, refused = [], []
    try:
        for waves in WAVES:
            for rows, prefetch, form in itertools.product(ROWS, (1, 0), FORMS[waves]):
                for name, v in (("waves", waves), ("rows", rows), ("prefetch", prefetch), ("form", form)):
                    ks.ks_set_option(name, v)
                try:
                    ms = _time(dtype, op, inclusive, d_in, d_out, steps, warmup)
                except ks.KsError as e:
                    if e.status != ks.KS_ERR_UNSUPPORTED:
                        raise
                    refused.append((waves, rows, prefetch, form))
                    continue
                results.append((ms, waves, rows, prefetch, form))
                print(f"waves={waves:2d} rows={rows:2d} prefetch={prefetch} form={form}: {ms:.4f} ms "
                      f"{nbytes / ms / 1e6:7.0f} GB/s (grid {ks.ks_get_option('last_grid')})", file=out, flush=True)
    finally:
        for name, v in (("waves", 0), ("rows", 0), ("prefetch", -1), ("form", -1)):
            ks.ks_set_option(name, v)
    default_ms = _time(dtype, op, inclusive, d_in, d_out, steps, warmup)
    results.sort()
    print(f"\n({dtype}, {op}) n={n} {'inclusive' if inclusive else 'exclusive'}: best first", file=out)
    for ms, waves, rows, prefetch, form in results[:10]:
        print(f"  {nbytes / ms / 1e6:7.0f} GB/s  waves={waves} rows={rows} prefetch={prefetch} form={form}", file=out)
    print(f"  {nbytes / default_ms / 1e6:7.0f} GB/s  library default", file=out)
    print(f"  refused as not fitting: {len(refused)} of {len(refused) + len(results)} combinations", file=out)
    return results


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--dtype", default="f32", choices=sorted(ks.DTYPES))
    ap.add_argument("--op", default="sum", choices=sorted(ks.OPS))
    ap.add_argument("--log2n", type=int, default=28)
    ap.add_argument("--n", type=int, default=0, help="element count (overrides --log2n)")
    ap.add_argument("--exclusive", action="store_true")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--random", action="store_true")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("tune needs a GPU", file=sys.stderr)
        return 2
    if not ks.ks_pair_supported(args.dtype, args.op):
        print(f"({args.dtype}, {args.op}) is not an instantiated pair", file=sys.stderr)
        return 2
    n = args.n if args.n > 0 else 1 << args.log2n
    search(args.dtype, args.op, n, not args.exclusive, args.steps, args.warmup, args.random)
    return 0


if __name__ == "__main__":
    sys.exit(main())
