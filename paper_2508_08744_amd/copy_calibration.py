"""A plain device-to-device copy of known size (1 GiB, three times), for calibrating what the
rocprofv3 FETCH_SIZE / WRITE_SIZE counters report per byte of HBM traffic on this machine:

    rocprofv3 --pmc FETCH_SIZE -- python3 paper_2508_08744_amd/copy_calibration.py
"""
import torch

if __name__ == "__main__":
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(3):
        a.copy_(b)
    torch.cuda.synchronize()
    print("copied 3 x %d bytes" % (a.numel() * 4))
