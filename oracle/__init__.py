"""CPU oracle for the ChunkWise LoRA hot path -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the bench's cpu_baseline leg may import this package; the
product package never does, and this package never imports the product.  See ``cwl_ref.c`` for
the arithmetic and ``reference.py`` for the numpy-facing wrapper.
"""
from .reference import (  # noqa: F401
    build,
    entropy,
    quantise,
    quantise_threshold,
    partition,
    select,
    linear,
    StreamState,
    stream_step,
    gated_linear,
    compose_scores,
    limit_high,
    bucket_sequences,
    partition_aligned,
    BucketState,
    stream_step_aligned,
    build_ladder,
    num_threads,
    set_num_threads,
    bf16_round,
    kv_quantise,
    kv_dequantise,
    SLOT_ABSENT,
)
