"""ONES evolutionary search (arXiv 2108.03645, Section 3.2) on MI355X: Python binding of
the C-ABI library plus the seeded synthetic clusters it is measured on."""
from . import workloads  # noqa: F401

__all__ = ["workloads", "ones"]


def __getattr__(name):
    if name == "ones":
        import importlib
        return importlib.import_module(".ones", __name__)
    raise AttributeError(name)
