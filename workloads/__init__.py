"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds configuration records, the weight/prompt generators and the
bf16 storage rounding.  It contains none of the method's arithmetic (no model
forward, no sampling, no verifier): both sides import it so that they see the
same numbers, and neither side imports the other.

The paper evaluates on trained checkpoints (GPT-2 small/XL, GPT-Neo, Vicuna
68M/7B; Sec. 4 "Dataset and Model Architecture") and on text prompts; neither
is available here, so the generators below produce random-init weights of the
same shapes and i.i.d. token-id prompts (uniform or Zipf) that stand in for them.
"""
from .configs import (ModelCfg, SprinterCfg, ARCH_GPT, ARCH_LLAMA, DT_F32, DT_BF16,
                      CTX_OWN_HISTORY, CTX_FULL_PREFIX, REJECT_REPLACE, REJECT_SD, config, mini_config, CONFIG_NAMES)
from .synth import (round_bf16, make_model_weights, make_verifier_weights,
                    make_weights, make_prompts, zipf_probs, model_weight_shapes,
                    verifier_weight_shapes)
from .calibrate import shifted_bias, logit
