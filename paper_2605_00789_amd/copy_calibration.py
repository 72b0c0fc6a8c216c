"""Plain device-to-device copies of known size (64 MiB and 512 MiB, four each).  Run under
`rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` to see what those counters report for a kernel whose HBM
traffic is known (reads N bytes, writes N bytes); the ratio scales the counters of the LightKV kernels."""
import torch

if __name__ == "__main__":
    for mib in (64, 512):
        a = torch.empty(mib * 1024 * 1024 // 2, dtype=torch.bfloat16, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(4):
            b.copy_(a)
        torch.cuda.synchronize()
