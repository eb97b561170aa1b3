"""MI355X-native sparse-embedding hot path (dedup, route, lookup forward/backward, row-wise Adagrad).

``paper_2604_06956_amd.binding`` is the thin Python layer over the C-ABI HIP library;
``paper_2604_06956_amd.workloads`` generates seeded synthetic inputs.  Importing the package
loads neither torch nor the HIP library; ``binding`` does both and fails loudly if the
library has not been built.
"""
__all__ = ["binding", "workloads", "build"]
