"""MI355X-native HE secure-aggregation hot path (FedML-HE, Algorithm 1).

The compute path lives in the HIP library under csrc/ (C ABI declared in
include/he_fedavg.h); `paper_2303_10837_amd.binding` is the thin ctypes layer
over it.  Nothing here falls back to a CPU implementation: if the library is
not built the binding raises.
"""
