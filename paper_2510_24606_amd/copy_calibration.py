"""A plain 1 GiB device-to-device copy, used to calibrate the rocprofv3 derived
counters FETCH_SIZE and WRITE_SIZE (KiB per dispatch): run it under
`rocprofv3 --pmc FETCH_SIZE` (then `--pmc WRITE_SIZE`) and divide the known
1 048 576 KiB by what the counter reports for the copy kernel."""
import torch


def main() -> None:
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()   # 1 GiB
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)          # reads 1 GiB, writes 1 GiB per launch
    torch.cuda.synchronize()


if __name__ == "__main__":
    main()
