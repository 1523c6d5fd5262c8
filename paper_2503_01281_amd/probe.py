"""Memory rates of this machine, as the access-bound kernels of the path see them.

    python -m paper_2503_01281_amd.probe [--gib 8] [--host-gib 8]

Runs dci_probe_read (streaming and random reads of several granules, with the lanes of a granule adjacent,
scrambled or spread over the wavefront) over a device buffer and over pinned host memory read by zero-copy,
plus one pinned host -> device copy, and prints a table.  Measurement only: nothing of the method is here.
"""
from __future__ import annotations

import argparse

import torch

from .binding import Context, dci_probe_read, pinned_empty


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=int, default=8, help="size of the device buffer")
    ap.add_argument("--host-gib", type=int, default=8, help="size of the pinned host buffer")
    args = ap.parse_args()
    ctx = Context(0)
    gib = 1 << 30
    dev = torch.empty(args.gib * gib, dtype=torch.uint8, device="cuda")
    dev.fill_(1)
    host = pinned_empty(args.host_gib * gib, torch.uint8)
    host.fill_(1)
    torch.cuda.synchronize()

    def run(name, mem, granule, n, order=0, wg=4096, nbytes=None):
        dci_probe_read(ctx, mem, granule, n, order, wg, 7, nbytes)
        ms = min(dci_probe_read(ctx, mem, granule, n, order, wg, 8 + k, nbytes) for k in range(3))
        if granule == 0:
            b = nbytes or mem.numel()
            print(f"{name:30s} streaming read, {wg:5d} workgroups          {b / ms / 1e6:9.1f} GB/s  ({ms:.3f} ms)", flush=True)
        else:
            g = abs(granule)
            how = {0: "adjacent lanes, in order", 1: "adjacent lanes, scrambled", 2: "lanes spread over the wavefront"}[order]
            lanes = "8 x 8 B" if granule < 0 else (f"{g} B" if g <= 16 else f"{g // 16} x 16 B")
            print(f"{name:30s} random {g:4d} B ({lanes:9s}; {how:32s}) {n / ms / 1e6:8.3f} G/s {n * g / ms / 1e6:9.1f} GB/s ({ms:.3f} ms)",
                  flush=True)

    run("HBM", dev, 0, 0)
    for g in (8, 16, 32, 64, 128, 256):
        run("HBM", dev, g, 1 << 26)
    for order in (0, 1, 2):
        run("HBM", dev, -64, 1 << 25, order)
    run("HBM, 256 MiB region", dev, 64, 1 << 26, nbytes=256 << 20)
    hb = min(2 * gib, host.numel())
    for wg in (4096, 1024, 256):
        run("pinned host (zero-copy)", host, 0, 0, wg=wg, nbytes=hb)
    for g in (8, 16, 32, 64, 128, 256, 512):
        run("pinned host (zero-copy)", host, g, 1 << 21)
    for wg in (256, 8192):
        run(f"pinned host, {wg} workgroups", host, 64, 1 << 21, 0, wg)
    for order in (0, 1, 2):
        run("pinned host (zero-copy)", host, -64, 1 << 21, order)
    run("pinned host (zero-copy)", host, 128, 1 << 21, 2)
    d = torch.empty(gib, dtype=torch.uint8, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    d.copy_(host[:gib], non_blocking=True)
    torch.cuda.synchronize()
    ev[0].record()
    d.copy_(host[:gib], non_blocking=True)
    ev[1].record()
    torch.cuda.synchronize()
    print(f"{'pinned host -> HBM copy':30s} hipMemcpyAsync, 1 GiB                    {gib / ev[0].elapsed_time(ev[1]) / 1e6:9.1f} GB/s", flush=True)


if __name__ == "__main__":
    main()
