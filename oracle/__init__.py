"""CPU oracle of the SPECS scoring + SubSample path. TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy code written from the paper's definitions. Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product path never does.
It imports nothing from the HIP package and shares no code with it.
"""
from .rounding import round_bf16, operand, float_accumulation_jitter
from .transformer import (linear, token_logprob, silu, log_softmax, rms_norm, rope, swiglu_ffn, attention, forward_sequences,
                          block_logprobs_full, reward_full, prefill, score_cached, PrefixCache)
from .subsample import scores, selection_probs, subsample, subsample_batch
from . import smc
from .generate import generate_blocks, sample_token
