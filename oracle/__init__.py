"""TEST INFRASTRUCTURE: plain CPU oracle of the estimate / drop / compaction path.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It shares nothing with the GPU library.
"""
from .reference import (VARIANT_BACK, VARIANT_FULL, VARIANT_LOWER, VARIANT_SF, VARIANT_UPPER,  # noqa: F401
                        build_oracle, clipper_drop, compact, estimate_drop, expand_paths, nexus_drop, priority_modes, queue_delay, run, stage_cost,
                        sub_latency)
