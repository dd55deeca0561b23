"""Device-resident mini-batch construction for sampling-based GNN training on MI355X.

`paper_2605_29346_amd.zg` is the thin ctypes binding over the C-ABI library (loaded on
first use; it raises if the library has not been built).  `paper_2605_29346_amd.workloads`
holds the seeded synthetic input generators and needs no GPU.
"""
__all__ = ["workloads", "zg"]
