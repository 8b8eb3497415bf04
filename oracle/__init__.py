"""fp64 CPU oracle (test infrastructure only; see glm_oracle.c for what it computes).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the GPU library and does not import it."""
from .loader import (  # noqa: F401
    build,
    attention,
    attention_rows,
    attention_weights,
    fork_copy,
    gather,
    kv_append,
    gather_tokens,
    lib_path,
)
