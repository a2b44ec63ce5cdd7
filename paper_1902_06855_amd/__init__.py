"""MI355X-native GradientFlow gradient-aggregation hot path (arxiv 1902.06855).

`paper_1902_06855_amd.workloads` holds the seeded synthetic input generators and
imports nothing else from this package.  `paper_1902_06855_amd.gf` is the thin
binding over the C-ABI library built from `csrc/`; it is imported on first use
so that the input generators stay usable where the HIP library is not built.
"""

__all__ = ["workloads", "gf"]


def __getattr__(name):
    if name in ("gf", "workloads"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
