"""L1 fill rate of a compute unit, measured with the library's probe kernel (vvs_debug_fill_probe).

    python -m paper_2511_13587_amd.fillrate

Bytes through the L1 of a CU = region x repetitions.  Three sources: one 1 MiB region read by every workgroup over and over
(it stays in the L2 of every XCD); a region of 1 MiB of its own per workgroup, read 8 times (256 MiB in all: beyond the L2s,
inside the 256 MB memory-side cache); 8 MiB of its own per workgroup, read once (2 GiB in all: from HBM).  The table gives
GB/s per workgroup (= per CU while there are at most 256 workgroups) for register loads and for direct-to-LDS loads."""
import sys

import torch

from . import binding as vb, synth


def main():
    ctx = vb.Context(vb.make_config(synth.TINY))
    dev = ctx.device
    src = torch.zeros(2 << 28, dtype=torch.int32, device=dev)          # 2 GiB
    print("source                      mode       workgroups waves   us/launch  GB/s per workgroup  TB/s all")
    cases = (("L2: one 1 MiB region", 1 << 20, 0, 64), ("own 1 MiB each, 8 times", 1 << 20, 1 << 20, 8), ("HBM: own 8 MiB each, once", 8 << 20, 8 << 20, 1))
    for label, region, stride, reps in cases:
        for mode, name in ((0, "registers"), (1, "to LDS")):
            for wgs in (64, 256):
                for waves in (4, 8, 16):
                    for _ in range(2):
                        ctx.vvs_debug_fill_probe(src, reps, mode, wgs, waves, region, stride)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    n = 5
                    e0.record()
                    for _ in range(n):
                        ctx.vvs_debug_fill_probe(src, reps, mode, wgs, waves, region, stride)
                    e1.record()
                    torch.cuda.synchronize()
                    t = e0.elapsed_time(e1) / n * 1e-3
                    per = region * reps / t / 1e9
                    print(f"{label:27s} {name:10s} {wgs:8d} {waves:6d} {t * 1e6:10.1f} {per:14.1f} {per * wgs / 1e3:14.2f}", flush=True)
    ctx.close()


if __name__ == "__main__":
    sys.exit(main())
