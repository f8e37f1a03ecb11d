"""MI355X-native hot path of CachedAttention (arXiv 2403.19708): thin Python binding over the
C ABI in include/ca.h, and over the placement manager in include/ca_store.h (module `store`).  All
computation happens in the library; this package only marshals arguments.  Importing it does not load the library; the first call does, and fails loudly if the
library has not been built (python -m paper_2403_19708_amd.build)."""
from .binding import (  # noqa: F401
    CaError,
    Config,
    Context,
    batch_validate,
    config_validate,
    lib_path,
    load_library,
    pointer_array,
    truncate_plan,
    tier_compact,
    truncate_plan_sinks,
)
