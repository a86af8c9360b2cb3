"""MI355X-native Tri-Accel optimizer step (arXiv 2508.16905): hand-written gfx950 kernels behind
a C ABI (``include/triaccel.h``), with a ctypes binding of the same names.

Importing this package loads nothing; the HIP library is loaded on first use and its absence is
an error (there is no CPU path in the product).
"""

from .binding import (  # noqa: F401
    BF16,
    FP16,
    FP32,
    STAGE_NAMES,
    Config,
    LayerInfo,
    PowerInfo,
    PowerTensor,
    StepArgs,
    StepResult,
    Tensor,
    TriAccelError,
    load_library,
    triaccel_batch_next,
    triaccel_cast_f32,
    triaccel_destroy,
    triaccel_get_state,
    triaccel_set_state,
    triaccel_init,
    triaccel_layer_state,
    triaccel_power_iter,
    triaccel_power_iter_static,
    triaccel_power_state,
    triaccel_power_times_get,
    triaccel_result,
    triaccel_set_graph,
    triaccel_set_profiling,
    triaccel_stage_times_get,
    triaccel_step,
    triaccel_strerror,
)
from .optimizer import TriAccel  # noqa: F401
