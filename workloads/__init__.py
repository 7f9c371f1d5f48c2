"""Seeded synthetic workload generators shared by the oracle tests and the GPU tests."""
from .generate import (  # noqa: F401
    BASE_SEED, HEAD_DIM, PAGE_SIZE, Workload, bf16_bits_to_f32, f32_to_bf16_bits,
    config1_tiny, config2_rag_fixed, config3_rag_zipf, config4_long_context, config5_128k,
    make_contexts, make_conversation, make_uniform, normal_bf16, probe_short_extend, rag_batch_from_blocks, rag_zipf_picks,
    sample_rows,
)
