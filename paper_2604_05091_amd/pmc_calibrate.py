"""Counter calibration run for HBM-traffic measurements.

    rocprofv3 --pmc FETCH_SIZE  -d <dir> --output-format csv -- python3 paper_2604_05091_amd/pmc_calibrate.py
    rocprofv3 --pmc WRITE_SIZE  -d <dir> --output-format csv -- python3 paper_2604_05091_amd/pmc_calibrate.py

Launches (1) a plain device-to-device copy kernel of a known size (1 GiB read + 1 GiB written) and
(2) one bf16 GEMM of the 7B QKV-projection shape through the C ABI, so that what FETCH_SIZE /
WRITE_SIZE read for the copy gives the scale factor for every other kernel's counters.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import torch  # noqa: E402

import paper_2604_05091_amd as mt  # noqa: E402


def main():
    L = mt.lib()
    n = 1 << 30
    src = torch.ones(n // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    M, N, K = 65536, 12288, 4096
    A = torch.randn((M, K), device="cuda").to(torch.bfloat16)
    B = torch.randn((N, K), device="cuda").to(torch.bfloat16)
    C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
    for _ in range(3):
        assert L.mt_k_gemm_nt(A.data_ptr(), K, B.data_ptr(), K, C.data_ptr(), N, None, 0, M, N, K, 0, 0, None) == 0
    torch.cuda.synchronize()
    print(f"copy: {n} bytes read + {n} bytes written per launch; gemm {M}x{N}x{K}: "
          f"algorithmic {2*(M*K+N*K)} bytes read, {2*M*N} bytes written")


if __name__ == "__main__":
    main()
