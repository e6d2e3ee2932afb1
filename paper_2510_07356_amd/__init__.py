"""GQA decode-step attention for MI355X (gfx950): split-KV partial kernel,
log-sum-exp combine kernel and paged block-table gather behind a C-ABI library.

`workloads` (numpy only) builds the seeded synthetic inputs; `binding` loads
the HIP library and marshals torch device pointers into it.  The binding is
imported on first use so that the input generators work without the library.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
