"""CPU float64 oracle for the SkipKV sentence-level KV-cache compression step.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import, call or link
anything in this package: only the test-suite, the smoke check and the
benchmark's ``cpu_baseline`` leg do.  It shares no code with the HIP kernels.
"""
from .skipkv_oracle import (  # noqa: F401
    token_importance,
    token_redundancy,
    token_scores,
    select_tokens,
    sentence_embeddings,
    sentence_redundancy,
    sentence_scores,
    select_sentences,
    remap_ranges,
    append_ranges,
    surviving_sentence_ids,
    append_sentence_ids,
    compact,
    compress_head,
    steer_add,
    steer_strength,
    round_to_bf16,
)
