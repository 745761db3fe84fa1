"""Launch the library's plain copy kernel on a buffer of known size (256 MiB, three times).

Run under `rocprofv3 --pmc FETCH_SIZE` (and again with WRITE_SIZE): the counter value of a k_plain_copy dispatch,
divided into 262144 KiB, is the factor by which the same counter has to be scaled for the HiRE kernels.

    rocprofv3 --pmc FETCH_SIZE -d out -o copy --output-format csv -- python3 -m paper_2402_09360_amd.pmc_calibrate
"""
import torch

from . import hire

if __name__ == "__main__":
    n = 256 << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        hire.hire_debug_plain_copy(src, dst)
    torch.cuda.synchronize()
    print(f"copied {n} bytes x3")
