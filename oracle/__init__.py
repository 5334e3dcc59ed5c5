"""fp64 CPU oracle of the SABlock compression path -- TEST INFRASTRUCTURE ONLY.

Nothing under this folder is part of the product: only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may import it.  It shares no
code with the HIP library and does not import the product package.
"""

from .sablock_ref import (  # noqa: F401
    build,
    score,
    score_layer,
    refine,
    search_blocks,
    select,
    compact,
    segment_score,
    pipeline_head,
    segment,
    decode_attention,
    window_attention,
)
