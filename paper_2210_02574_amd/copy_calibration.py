"""Plain device-to-device copy of 256 MiB, five launches: the reference against which the HBM traffic counters
of the profiler are scaled (`rocprofv3 --pmc FETCH_SIZE -- python3 paper_2210_02574_amd/copy_calibration.py`,
then the same with WRITE_SIZE).  The copy reads and writes exactly 262144 KiB per launch."""
import torch


def main():
    a = torch.empty(32 * 1024 * 1024, dtype=torch.int64, device="cuda").random_()
    b = torch.empty_like(a)
    for _ in range(5):
        b.copy_(a)
    torch.cuda.synchronize()
    print("copied 5 x 256 MiB")


if __name__ == "__main__":
    main()
