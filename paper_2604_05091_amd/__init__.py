"""MI355X-native streamed transformer training step (MegaTrain's per-layer streaming, Algorithm 1).

The product is the C-ABI library `libmegatrain_mi355.so` (HIP kernels + stream/event scheduler +
host Adam); this package is its thin ctypes binding.  There is no CPU fallback: if the library is
missing or no GPU is present, the calls that need one fail loudly.
"""
from .binding import (  # noqa: F401
    MtError, ModelCfg, Stats, TrainHandle, lib, lib_path, link_probe, device_count, device_synchronize, model_flops, STATUS_NAMES,
    FLAG_SERIAL, FLAG_COMPUTE_ONLY, FLAG_COPY_ONLY, FLAG_KERNEL_TIMING, FLAG_GRAD_SLABS, FLAG_STAGED_WEIGHTS,
)
