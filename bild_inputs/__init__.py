"""Seeded synthetic inputs shared by the CPU oracle and the HIP library:
model-pair shapes, weights and token ids.  Holds no model arithmetic."""
from .configs import (ACT_GATED_GELU, ACT_RELU, ACT_SWIGLU, DT_BF16, DT_F32, PAIRS, POS_RELATIVE, POS_ROPE,
                      POS_SINUSOIDAL, ModelShape, PairConfig, llama_pair, mt5_pair, t5_pair, tiny_pair,
                      toy_pair)
from .generate import (make_pair_weights, make_source, make_tokens, make_uniforms, make_weights, tensor_names,
                       tensor_shape, to_bf16_values, truncate_weights)
