"""Seeded synthetic inputs for the sparse-drafter hot path.

This package only *creates data*: random bf16 weights with a fixed pruning
pattern, random bf16 activations, and random draft/target token ids.  It holds
none of the arithmetic of the method (no linear, no packing, no verification)
and is the only code shared by the CPU oracle and the HIP path.

The stand-ins follow the shapes of the drafters the paper evaluates (Sec. 3,
Llama-3.2 / Qwen-2.5 decoder blocks with every decoder linear pruned, embedding
and LM head left dense); real checkpoints and evaluation prompts are not used.
"""

from .gen import (  # noqa: F401
    SEED,
    PROJ,
    CONFIGS,
    StackShape,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    n_keep,
    magnitude_mask_per_row,
    magnitude_mask_global,
    mask_2of4,
    gen_weight,
    gen_weight_dense,
    gen_x,
    gen_verify,
    gen_lm_head,
    gen_final_hidden,
    gen_kv_history,
    stack_matrices,
    layer_matrix_shapes,
)
