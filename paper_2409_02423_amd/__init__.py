"""zc: fixed-rate block-transform compression of collective message buffers
for MI355X (gfx950).  The codec runs in hand-written HIP kernels behind a C ABI
(include/zc.h); `paper_2409_02423_amd.zc` is the thin Python binding and
`paper_2409_02423_amd.workloads` generates synthetic message buffers."""

__all__ = ["zc", "workloads"]
