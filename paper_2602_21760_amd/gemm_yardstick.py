"""Yardstick for the bf16 MFMA GEMM (a measurement aid, not part of the hot path): times hyb_linear next to the vendor
GEMM library (through torch.matmul) on the four GEMM shapes of the SD3-shaped joint block and on a large square
problem, with N(0, 1) data and with all-zero data.  All-zero operands draw far less power, so the ratio of the two
says how much of a kernel's rate on real data is set by the chip's power management rather than by the kernel."""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))  # repo root
import torch

from paper_2602_21760_amd import binding as hb


def _time(fn, iters=20):
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1000 / iters


def main():
    hb.lib()
    print("| m | n | k | data | hyb_linear us | TFLOP/s | vendor library us | TFLOP/s |")
    print("|---|---|---|---|---|---|---|---|")
    for m, n, k in ((4429, 4608, 1536), (4429, 1536, 1536), (4429, 6144, 1536), (4429, 1536, 6144), (8192, 8192, 8192)):
        for data in ("normal", "zeros"):
            if data == "normal":
                a = torch.randn(m, k, device="cuda").to(torch.bfloat16)
                w = (0.02 * torch.randn(n, k, device="cuda")).to(torch.bfloat16)
            else:
                a = torch.zeros(m, k, device="cuda", dtype=torch.bfloat16)
                w = torch.zeros(n, k, device="cuda", dtype=torch.bfloat16)
            out = torch.empty(m, n, device="cuda", dtype=torch.bfloat16)
            t_h = _time(lambda: hb.hyb_linear(a, w, None, out))
            t_v = _time(lambda: torch.matmul(a, w.t(), out=out))
            fl = 2.0 * m * n * k / 1e6
            print("| %d | %d | %d | %s | %.1f | %.0f | %.1f | %.0f |" % (m, n, k, data, t_h, fl / t_h, t_v, fl / t_v), flush=True)


if __name__ == "__main__":
    main()
