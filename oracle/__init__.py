"""Plain CPU oracle of the rollout hot path.  TEST INFRASTRUCTURE ONLY: imported by tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg, never by the product path."""
from .model import (OracleModel, ContiguousKV, PagedKV, rmsnorm, rope, rope_cos_sin, softmax, silu,
                    gqa_attention, paged_decode_attention, greedy_token, log_prob)
from .scheduler import (OracleRollout, Seq, splitmix64_permutation, QUEUED, ACTIVE, FINISHED, HARVESTED,
                        MODE_PARTIAL, MODE_ONPOLICY, MODE_SYNC, EOS_FORCED_ONLY, EOS_NATURAL_OR_FORCED)
from .sampling import philox4x32_10, uniforms, perturbed_scores, sample_token, log_prob_at
