"""CPU oracle for the `pred` hot path: TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct NumPy code written from the paper's description of
`pred` (section 4.1) and of the KV-cache file system KVFS (section 4.2).  It shares no
code with the HIP library and never imports it.  Only tests, the smoke check and the
benchmark's `cpu_baseline` leg may import this package; the product path never does.

Pin status: every function here is pinned by CPU tests against closed forms, brute
force, invariants and a library routine (see tests/test_oracle_*.py); nothing in this
package is "parity unpinned".
"""
from .kvfs_model import KVFSModel, KVError, PagePool  # noqa: F401
from .attention import gather_file, dense_attention, pred_batch  # noqa: F401
