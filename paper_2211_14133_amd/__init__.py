"""MI355X-native K-FAC work items (curvature, inversion, precondition) behind a C ABI."""
from .binding import (  # noqa: F401
    InvertPlan,
    KfacError,
    kfac_assign_work,
    kfac_perf_model,
    kfac_mfma_probe,
    kfac_curvature,
    kfac_curvature_grouped,
    kfac_curvature_grouped_workspace,
    kfac_invert,
    kfac_invert_batched,
    kfac_invert_noalloc,
    kfac_invert_batched_workspace,
    kfac_precondition,
    kfac_precondition_grouped,
    kfac_precondition_grouped_workspace,
    load,
)
