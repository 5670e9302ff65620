"""A plain device-to-device copy of known size, used to calibrate rocprofv3's HBM byte counters.

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2109_09868_amd.copy_probe
    rocprofv3 --pmc WRITE_SIZE -- python3 -m paper_2109_09868_amd.copy_probe

Each of the REPS copy kernels reads SIZE_BYTES and writes SIZE_BYTES; the ratio between SIZE_BYTES
and what the counter reports for one of them is the factor applied to the counter's reading for the
library's kernels.  The buffers are far larger than the 256 MB last-level cache.
"""
import torch

SIZE_BYTES = 2 << 30
REPS = 4


def main():
    dev = torch.device("cuda:0")
    src = torch.empty(SIZE_BYTES // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(REPS):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d bytes x %d" % (SIZE_BYTES, REPS))


if __name__ == "__main__":
    main()
