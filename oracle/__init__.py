"""fp64 CPU oracle of the cached-prefill path.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It never imports the HIP library's package, and that package never imports
this one.
"""
from .ca_oracle import (  # noqa: F401
    attention_positions,
    build,
    cached_attention,
    cached_attention_kept,
    compact_tier,
    kept_indices_sinks,
    kv_bytes_per_token,
    n_threads,
    pack,
    rebase,
    rope,
    truncate_plan,
    unpack,
)
