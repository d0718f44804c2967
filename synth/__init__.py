"""Seeded synthetic inputs (model weights, prompts, draft blocks).

This package only *generates inputs*.  It holds none of the method's
arithmetic (no transformer forward, no accept logic) and imports neither the
CPU oracle nor the HIP package, so both sides may be fed from it.
"""
from .model import (  # noqa: F401
    EEConfig, TENSOR_IDS, tiny_config, llama8b_config, llama70b_config,
    tensor_shape, gen_tensor, gen_tensor_rows, WeightStore, f32_to_bf16_bits,
    bf16_bits_to_f32,
)
from .workload import (  # noqa: F401
    gen_prompt, gen_context_lengths, draw_first_mismatch, make_draft_block,
    expected_accept_len,
)
