"""MI355X-native draft-tree verification (READER, arXiv 2508.09072).

`workloads` draws synthetic inputs; `binding` wraps the C-ABI HIP library
(`reader_tree_attn`, `reader_accept_path`, `reader_kv_compact`).  The binding is
imported lazily so that the input generator can be used without the library.
"""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in ("workloads", "binding"):
        import importlib
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
