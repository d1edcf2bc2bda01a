"""MI355X-native hot path of Symphony's `pred` system call: batched attention over the
paged, copy-on-write KV-cache file system (paper sections 4.1, 4.2, 4.4).

`synth` holds the seeded workload generators (no method arithmetic); `binding` is the thin
ctypes layer over the C-ABI library `libsymphony_kv.so` built from `csrc/`.  Importing the
package does not load the library; the first call that needs it does, and raises if it has
not been built.
"""
from . import synth  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
