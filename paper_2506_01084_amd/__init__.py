"""zip2zip dynamic-vocabulary hot path for AMD MI355X (gfx950).

`workloads` (seeded synthetic inputs) imports without the HIP library; the
binding in `api` loads the C-ABI shared library on first use and raises if it
is missing -- there is no CPU fallback.
"""
__all__ = ["workloads", "api"]
