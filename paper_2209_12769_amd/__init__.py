"""MI355X-native batched evaluation of fusion candidates (graph contraction +
GNN cost model) behind the C ABI of include/disco.h.  Nothing is loaded at
import time; `binding.lib()` loads libdisco.so and raises if it is missing."""
__all__ = ["binding", "workloads", "build"]
