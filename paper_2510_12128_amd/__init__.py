"""MI355X-native nuGPR marginal-log-likelihood hot path (HIP kernels behind a C ABI).

`binding` wraps libnugpr.so (argument marshalling only); `inputs` holds the seeded
synthetic input generators; `build` compiles the library in-tree.  Importing this
package does not load the library; the first call into `binding` does, and fails loudly
when it is missing.
"""
from . import inputs  # noqa: F401
from .binding import (  # noqa: F401
    Context, NugprError, lib_path, load_library,
    NUGPR_OK, NUGPR_NOT_PD, NUGPR_INDEFINITE, NUGPR_NOT_CONVERGED,
    NUGPR_ERR_INVALID, NUGPR_ERR_WORKSPACE, NUGPR_ERR_HIP, NUGPR_ERR_STATE, NUGPR_ISOTROPIC,
)
