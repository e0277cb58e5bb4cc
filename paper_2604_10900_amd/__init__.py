"""MI355X-native CASK compression event: HIP kernels behind a C ABI plus a thin binding."""
from .binding import (BF16, F32, Batch, CaskError, Outputs, Params, attend, compress, compress_static, compress_step, consolidate,
                      group_diagnostics, load, mass_diagnostics, partition, plan, prefix_evict, score,
                      workspace_bytes)

__all__ = ["BF16", "F32", "Batch", "CaskError", "Outputs", "Params", "attend", "compress", "compress_static", "compress_step",
           "consolidate", "group_diagnostics", "load", "mass_diagnostics", "partition", "plan", "prefix_evict",
           "score", "workspace_bytes"]
