"""Plain device-to-device copy of a known size, used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE
counters: run it under the same --pmc command as bench.py and divide the counter it shows for the
copy kernel by the bytes printed here.

    rocprofv3 --pmc FETCH_SIZE -d out -o calib -- python3 paper_1712_01670_amd/traffic_calib.py
"""
import torch

if __name__ == "__main__":
    n = 256 * 1024 * 1024
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copy kernel: {n} bytes read, {n} bytes written per launch")
