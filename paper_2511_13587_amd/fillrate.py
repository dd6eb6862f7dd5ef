"""L1 fill rate of a compute unit, measured with the library's probe kernel (vvs_debug_fill_probe).

    python -m paper_2511_13587_amd.fillrate

Every workgroup reads the same region over and over (1 MiB: it stays in the L2 of every XCD; 256 MiB: it comes from
HBM), so bytes through the L1 of a CU = region x repetitions; the table gives GB/s per workgroup (= per CU while there
are at most 256 workgroups) for register loads and for direct-to-LDS loads, by workgroups and waves per workgroup."""
import sys

import numpy as np
import torch

from . import binding as vb, synth


def main():
    ctx = vb.Context(vb.make_config(synth.TINY))
    dev = ctx.device
    print("region  mode       workgroups waves   us/launch  GB/s per workgroup  TB/s all")
    for region_mib, reps in ((1, 64), (256, 1)):
        src = torch.from_numpy(np.random.default_rng(0).integers(0, 2**31 - 1, size=region_mib << 18, dtype=np.int32)).to(dev)
        for mode, name in ((0, "registers"), (1, "to LDS")):
            for wgs in (64, 256, 512):
                for waves in (4, 8, 16):
                    r = reps if region_mib == 1 else 1
                    for _ in range(2):
                        ctx.vvs_debug_fill_probe(src, r, mode, wgs, waves)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    n = 5
                    e0.record()
                    for _ in range(n):
                        ctx.vvs_debug_fill_probe(src, r, mode, wgs, waves)
                    e1.record()
                    torch.cuda.synchronize()
                    t = e0.elapsed_time(e1) / n * 1e-3
                    per = (region_mib << 20) * r / t / 1e9
                    print(f"{region_mib:4d} MiB {name:10s} {wgs:8d} {waves:6d} {t * 1e6:10.1f} {per:14.1f} {per * wgs / 1e3:14.2f}", flush=True)
        del src
    ctx.close()


if __name__ == "__main__":
    sys.exit(main())
