"""Runs the library's plain copy kernel on a buffer of known size, so that a profiler
run of this module (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) shows what the HBM traffic
counters read for a known number of bytes.  python -m paper_2406_17404_amd.copy_probe"""
import torch

from . import binding as b

GIB = 1 << 30


def main(nbytes: int = GIB, reps: int = 5) -> None:
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        b.trj_copy_probe(dst, src, nbytes)
    torch.cuda.synchronize()
    print(f"copied {nbytes} bytes x {reps}")


if __name__ == "__main__":
    main()
