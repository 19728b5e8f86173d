"""Plain device-to-device copy of a known size, used to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters.

    python3 -m paper_2502_16982_amd.copy_probe [--mib 1024] [--repeats 5]

Each repeat is one torch copy kernel that reads and writes exactly --mib MiB; comparing the counter values
rocprofv3 reports for it with that size gives the scale factor applied to the counters of the Muon kernels.
"""
import argparse
import json

import torch


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--repeats", type=int, default=5)
    args = ap.parse_args()
    n = args.mib * 2 ** 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.repeats):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes": n, "repeats": args.repeats}))


if __name__ == "__main__":
    main()
