"""Plain device-to-device copy of a known size, for calibrating HBM byte counters.

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2107_06925_amd.copy_probe

Streams 1 GiB (2^29 bf16 elements) three times through torch's elementwise
kernel dst = src + 1: each launch reads 1 GiB and writes 1 GiB of HBM.  (A
same-dtype copy_ would be a runtime memcpy, which the kernel counters do not see.)
"""
import torch

N = 1 << 29


def main():
    src = torch.ones(N, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1.0, out=dst)
    torch.cuda.synchronize()
    print("streamed", src.numel() * src.element_size(), "bytes in and out, x3")


if __name__ == "__main__":
    main()
