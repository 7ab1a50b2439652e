"""CPU oracle for the speculative-decoding hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct numpy code written from the paper's statement of
speculative sampling (Sec. 2, Preliminary), the EAGLE draft-model input (Sec. 2),
the dynamic draft tree's two knobs (appendix Drafting Hyper-Parameters) and the
lossless-acceptance statement (Sec. 4.1, Metrics).  Nothing here is shared with
the HIP path, and the product never imports this package: only tests, the smoke
check and the benchmark's cpu_baseline leg do.

Pin status (see tests/test_oracle_*.py):
  target forward, tree verify, greedy / rejection acceptance, rerank,
  compaction, RNG                      : pinned
  draft model architecture (fc + one pre-norm layer, no final norm, RoPE
  positions) and the expansion order   : parity unpinned by the paper; pinned
  only for self-consistency (incremental == full recompute) and through the
  property that ANY draft tree leaves the output unchanged.
"""
from .llama import Weights, KVCache, rmsnorm, rope, attention_row, decoder_layer, target_forward, draft_forward
from .rng import mix64, uniform01, gumbel
from .spec import (Tree, SpecState, greedy_decode, sample_decode, prefill, draft_tree, verify_tree, accept_greedy,
                   accept_sample, commit, spec_decode, log_softmax, top_k)
