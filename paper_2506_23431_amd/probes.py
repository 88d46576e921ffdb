#!/usr/bin/env python3
"""Device probes behind the design decisions: what a kernel that only reads reaches from HBM, from
the L2 caches and from the last-level cache, and how fast a SIMD issues matrix-core instructions
with one or more waves on it.

  python -m paper_2506_23431_amd.probes
"""

import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main(argv=None):
    import torch
    from paper_2506_23431_amd import binding
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    buf = torch.ones(1 << 30, dtype=torch.uint8, device=dev)       # 1 GiB
    out = {"hbm_stream": [], "slices": [], "mfma_issue": []}
    for mb in (8, 25, 34, 76, 131):
        gbs = binding.measure_read_bandwidth(buf.data_ptr(), buf.numel(), mb * 1000 * 1000 // 4096 * 4096, 200)
        out["hbm_stream"].append({"MB_per_launch": mb, "GB/s": gbs})
        print(f"plain read, {mb:4d} MB per launch, launches back to back: {gbs:8.0f} GB/s "
              f"({mb * 1e6 / gbs * 1e-3:5.1f} us per launch)", flush=True)
    for blocks, kib in ((256, 64), (512, 64), (256, 128), (1024, 64), (1024, 256)):
        gbs = binding.measure_cached_read_bandwidth(buf.data_ptr(), buf.numel(), blocks, kib * 1024, 64)
        out["slices"].append({"blocks": blocks, "slice_KiB": kib, "GB/s": gbs})
        print(f"{blocks:5d} blocks re-reading private slices of {kib:3d} KiB ({blocks * kib / 1024:6.1f} MB in all) "
              f"64 times: {gbs:8.0f} GB/s", flush=True)
    for waves in (1, 2, 4):
        ns = binding.measure_mfma_issue(buf.data_ptr(), buf.numel(), waves, 4096)
        out["mfma_issue"].append({"waves_per_simd": waves, "ns_per_instruction": ns})
        print(f"16x16x32 bf16 matrix-core instruction, {waves} wave(s) per SIMD: {ns:6.2f} ns per instruction and SIMD "
              f"= {ns * 2.4:5.1f} clocks at 2.4 GHz, {16384 / ns * 1024 * 1e-3:6.0f} TFLOP/s over 1024 SIMDs",
              flush=True)
    print(json.dumps(out))
    return out


if __name__ == "__main__":
    main()
