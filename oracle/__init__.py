"""CPU oracle for the PM-KVQ hot path -- TEST INFRASTRUCTURE, not a product path.

A plain, slow numpy implementation of what the HIP library computes: the asymmetric
group-wise quantizer (Sec. 2.2, Eq. 1-2), canonical bit packing, the Equivalent Right
Shift bit-width shrinking step (Sec. 3.1, Eq. 3, and the appendix theorem) with the two
alternative strategies of the ablation in Sec. 4.3.1 (Direct and Modified Right Shift), the
channel-wise reparameterization of Sec. 3.3 (Eq. 7-8: keys stored as K Lambda^-1, queries used as Q Lambda), the
block-wise memory allocation of Sec. 3.2 (sensitivity terms of Eq. 5 with the gradients as inputs, and the
integer program of Eq. 6 by enumeration and by the knapsack recurrence), the
progressive-quantization bookkeeping of Sec. 3.1 (with the 16-bit tier either raw fp16 values or, as an option, the
integer INT16 format of Sec. 4.1.2, from which 16 -> 8 is a step of Eq. 3 as well), and single-token GQA attention
in fp64 over the de-quantized cache.  It shares no code with the HIP path and imports nothing
from it; only tests, the smoke check and the bench's cpu_baseline leg may import it.

Pinned by tests/test_oracle_*.py against: the appendix theorem (exhaustively and in exact
rationals), round-trip error bounds, library fp64 attention on 16-bit caches, brute-force
loops on tiny caches, closed forms, the 4K/8K/16K shrink schedule of the appendix
"Analysis of Progressive Quantization", Table 1's byte counts, and the two properties
Sec. 4.3.1 states for the Direct (dynamic range kept) and Modified (bucket means) shifts;
the reparameterization by exactness for power-of-two factors, Q Lambda (K Lambda^-1)^T = Q K^T, and Eq. 8 on
hand-made keys; the allocation by enumeration against the recurrence, by its limiting cases (everything fits,
nothing fits, the uniform-2-bit-fits / uniform-4-bit-does-not situation of Sec. 3.2) and by a hand-solved instance;
the INT16 tier by exact-rational nearest-level checks, the clamp bound that the fp16 scale makes necessary, a
constructed family with exact scales on which Eq. 3 at b = 8 must reproduce the direct 8-bit codes element for
element, and the manual 16 -> 8 -> 4 chain on evicted window pages.

Parity unpinned: none of the functions here; the paper's accuracy tables are not reproduced.
"""
from .quantizer import (quantize, dequantize, pack_codes, unpack_codes, shrink_codes,
                        shrink_scale, shrink_step, bytes_per_token_head, LEVELS,
                        SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED,
                        calibrate_lambda, reparam_keys, reparam_queries, LAMBDA_FLOOR,
                        rope_rotate_keys)
from .attention import decode_attention_fp64
from .allocation import sensitivity, allocate_bits_bruteforce, allocate_bits_dp
from .cache import (OracleCache, CacheConfig, BudgetError, StateError, POLICY_PAPER, POLICY_OLDEST_FIRST,
                    TIER16_FP16, TIER16_INT16, decode_step_batch)

__all__ = ["quantize", "dequantize", "pack_codes", "unpack_codes", "shrink_codes", "shrink_scale", "shrink_step",
           "SHIFT_EQUIVALENT", "SHIFT_DIRECT", "SHIFT_MODIFIED", "calibrate_lambda", "reparam_keys",
           "reparam_queries", "LAMBDA_FLOOR", "sensitivity", "allocate_bits_bruteforce", "allocate_bits_dp", "rope_rotate_keys",
           "bytes_per_token_head", "LEVELS", "decode_attention_fp64", "OracleCache", "CacheConfig",
           "BudgetError", "StateError", "POLICY_PAPER", "POLICY_OLDEST_FIRST", "TIER16_FP16", "TIER16_INT16", "decode_step_batch"]
