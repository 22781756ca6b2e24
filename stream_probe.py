#!/usr/bin/env python3
"""Fill rate of a compute unit's L1 against the bytes it keeps in flight, for data that comes from L2, from
the memory-side cache and from HBM (development probe `coreinfer_dev_stream_probe` of the library).

    python3 stream_probe.py

Every workgroup streams 16-byte loads over a window, `depth` loads in flight per thread.  Printed per case:
bytes in flight per compute unit (threads x depth x 16 x workgroups per compute unit), time, aggregate rate
and rate per compute unit.  rate x latency = bytes actually outstanding: where the rate stops growing with
the bytes in flight, the L1's own limit of outstanding lines is reached."""

from __future__ import annotations

import torch

from paper_2410_18311_amd import coreinfer as ci

DEV = "cuda:0"
CUS = 256
PER_WG_BYTES = 32 << 20  # streamed by every workgroup per launch


def main():
    buf = torch.ones(5 << 29, dtype=torch.uint8, device=DEV)
    out = torch.zeros(4096, dtype=torch.int32, device=DEV)
    cases = [
        ("one 1 MB window shared by all workgroups (L2 hits)", 1 << 20, False),
        ("64 KB window per workgroup (L2 hits, nothing shared)", 64 << 10, True),
        ("one 64 MB window shared by all (memory-side cache)", 64 << 20, False),
        ("2 MB window per workgroup (HBM: 0.5 to 1 GB in all)", 2 << 20, True),
    ]
    shapes = [(256, 64, 2), (256, 64, 4), (256, 64, 8), (256, 128, 8), (256, 256, 8), (256, 512, 8), (256, 512, 16),
              (512, 512, 8), (512, 512, 16)]
    for name, win, per_wg in cases:
        print(f"-- {name}")
        for wgs, threads, depth in shapes:
            iters = PER_WG_BYTES // (threads * depth * 16)
            def launch():
                ci.dev_stream_probe(buf, win, per_wg, wgs, threads, depth, iters, out)
            launch()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            launch()
            launch()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) / 2 * 1e3
            total = wgs * iters * threads * depth * 16
            inflight = wgs / CUS * threads * depth * 16
            print(f"   {wgs:4d} workgroups x {threads:3d} threads x {depth:2d} loads: {inflight / 1024:6.1f} KB in flight per CU, "
                  f"{us:8.1f} us, {total / us / 1e6:6.2f} TB/s, {total / us / 1e3 / CUS:6.1f} GB/s per CU", flush=True)

    # the load stream of a 128-byte-wide operand tile: rows `pitch` bytes apart
    print("-- tile pattern: 256 threads, a load instruction = 128 bytes of each of 32 rows, 64 k-steps along the rows")
    for shared in (True, False):
        for pitch in (8192, 8192 + 128, 8192 + 256, 8192 + 1024, 10240, 18432):
            for depth in (8, 16):
                iters = 16384 // depth
                def launch():
                    ci.dev_tile_probe(buf, pitch, shared, CUS, depth, 64, iters, out)
                launch()
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                launch()
                launch()
                b.record()
                torch.cuda.synchronize()
                us = a.elapsed_time(b) / 2 * 1e3
                total = CUS * iters * depth * 4096
                print(f"   {'rows shared by all workgroups (L2 hits)' if shared else 'rows of its own per workgroup (HBM)  '}, pitch {pitch:6d}, "
                      f"{depth * 4:3d} KB in flight per CU: {us:8.1f} us, {total / us / 1e6:6.2f} TB/s, "
                      f"{total / us / 1e3 / CUS:6.1f} GB/s per CU", flush=True)

    # launches of the size of one decode layer: every byte read once, dependent launches replayed from a HIP graph
    print("-- read-only launches of a decode layer's size, 20 launches over different parts of the buffer in a HIP graph")
    for wgs, threads, depth in ((256, 512, 8), (512, 512, 8), (256, 512, 4)):
        for mb in (42, 85, 107, 141, 212, 425):
            per_iter = threads * depth * 16
            iters = max(1, mb * 1000000 // (wgs * per_iter))
            win = iters * per_iter
            nbytes = win * wgs
            regions = min(20, buf.numel() // nbytes)
            def layers():
                for r in range(regions):
                    ci.dev_stream_probe(buf[r * nbytes:(r + 1) * nbytes], win, True, wgs, threads, depth, iters, out)
            layers()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                layers()
            g.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                g.replay()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) / 10 / regions * 1e3
            print(f"   {wgs:4d} workgroups x {threads} threads x {depth} loads, {nbytes / 1e6:6.1f} MB per launch: {us:6.2f} us launch to launch, "
                  f"{nbytes / us / 1e6:5.2f} TB/s = {nbytes / us / 1e6 / 8:.3f} of 8 TB/s", flush=True)


if __name__ == "__main__":
    main()
