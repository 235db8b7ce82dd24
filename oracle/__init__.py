"""CPU oracles: fp64 tree attention and the cache bookkeeping after acceptance (test infrastructure only).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP path and never imports it.
"""
from .treeattn_oracle import (  # noqa: F401
    build_oracle,
    oracle_threads,
    tree_attn_oracle,
    tree_attn_oracle_sample,
)
from . import kv_compact_oracle  # noqa: F401,E402  (module: kv_compact_oracle.kv_compact_oracle)
