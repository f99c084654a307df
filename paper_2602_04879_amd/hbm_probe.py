"""Counter calibration and streaming ceiling: runs the library's plain copy kernel and read-only
kernel over buffers of known size.

  python3 -m paper_2602_04879_amd.hbm_probe [--gib 4] [--iters 10]

Under `rocprofv3 --pmc FETCH_SIZE` (then `--pmc WRITE_SIZE`) the copy kernel's counter per
dispatch, divided into the bytes it is known to move (`--gib` GiB read, `--gib` GiB written),
gives the factor that turns the same counter of a loss kernel into HBM bytes.  Run plainly it
prints the copy, read-only and write-only bandwidths (HIP events on the launch stream)."""
import argparse
import json

import torch

from . import binding as B


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=float, default=4.0)
    ap.add_argument("--iters", type=int, default=10)
    a = ap.parse_args()
    n = int(a.gib * (1 << 30)) // 16 * 16
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    s = torch.cuda.current_stream()
    out = {"bytes": n, "iters": a.iters}
    for name, fn in (("copy", lambda: B.probe_copy(dst, src, s)), ("read", lambda: B.probe_read(src, sink, s)),
                     ("fill", lambda: B.probe_fill(dst, 0x3c003c00, s))):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        for _ in range(a.iters):
            fn()
        e1.record(s)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / a.iters
        moved = 2 * n if name == "copy" else n
        out[name + "_ms"] = ms
        out[name + "_GBs"] = moved / (ms * 1e-3) / 1e9
        if name == "copy":
            assert torch.equal(src, dst)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
