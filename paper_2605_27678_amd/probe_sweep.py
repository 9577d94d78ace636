"""Prints how the HBM rate of a plain R-read : W-write streaming kernel depends
on the launch shape on this machine (hp_probe_stream with explicit shapes):
tile size x workgroup size x resident-wave cap.  Useful to see where the narrow
occupancy optimum sits before trusting the library defaults, and to compare
hp_forward / hp_backward against their access pattern's own ceiling.

    python -m paper_2605_27678_amd.probe_sweep --read 1 --write 4 --mb 400
"""
from __future__ import annotations

import argparse

from . import binding as hp


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--read", type=int, default=1, help="arrays read (0..8)")
    ap.add_argument("--write", type=int, default=4, help="arrays written (1..8)")
    ap.add_argument("--mb", type=int, default=400, help="megabytes per array")
    ap.add_argument("--nontemporal", type=int, default=None, help="bit 0 loads, bit 1 stores (default 2 if W>=R else 3)")
    args = ap.parse_args()
    nt = args.nontemporal if args.nontemporal is not None else (3 if args.read > args.write else 2)
    nbytes = args.mb * 1000000 // 4096 * 4096
    caps = [4, 6, 8, 12, 16, 24, 32]
    print(f"{args.read}R:{args.write}W, {nbytes} B per array, nontemporal={nt}; GB/s by resident waves per CU")
    print("tile_bytes block chunks/lane | " + " ".join(f"{c:>6d}" for c in caps))
    for tile in (1024, 2048, 4096, 8192, 32768):
        for block in (64, 128, 256, 1024):
            chunks = tile // 16 // block
            if chunks not in (1, 2, 4, 8, 32):
                continue
            row = []
            for cap in caps:
                if cap < 2 * (block // 64):
                    row.append("     -")
                    continue
                shape = dict(tile_bytes=tile, block_threads=block, waves_per_cu=0 if cap == 32 else cap, nontemporal=nt)
                gbps, _ = hp.hp_probe_stream(args.read, args.write, nbytes, shape)
                row.append(f"{gbps:6.0f}")
            print(f"{tile:10d} {block:5d} {chunks:11d} | " + " ".join(row), flush=True)
    best, shape = hp.hp_probe_stream(args.read, args.write, nbytes)
    print(f"best of the tuner's search space: {best:.0f} GB/s with {shape}")


if __name__ == "__main__":
    main()
