"""MI355X-native paged-KV decode attention and KV-block swap (gfx950 HIP kernels
behind a C ABI).  The compute API is in :mod:`paper_2602_07878_amd.binding`;
seeded synthetic inputs are in :mod:`paper_2602_07878_amd.workloads`.
Nothing is loaded at import time; the HIP library is opened on first use and a
missing library is an error, never a fallback."""

__all__ = ["binding", "workloads", "build"]
