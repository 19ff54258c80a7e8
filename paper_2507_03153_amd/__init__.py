"""MI355X-native HGCA decode-time hybrid attention (arXiv 2507.03153, Sec. 3.3).

`hgca`      -- ctypes binding of the C-ABI HIP library (needs torch + a GPU to run).
`workloads` -- seeded synthetic inputs (numpy only).
`build`     -- compiles the HIP library for gfx950 with hipcc.
"""
__all__ = ["hgca", "workloads", "build"]
