"""MI355X-native tile-sparse attention path (head-aware tiling, statistics-aware tile
scoring, per-query-tile top-k, block-sparse flash attention) behind a C-ABI library.

`paper_2605_30325_amd.veda` is the ctypes binding of libveda.so; `workloads` draws the
seeded synthetic inputs.  Importing the package loads nothing heavy."""
__all__ = ["veda", "workloads"]
