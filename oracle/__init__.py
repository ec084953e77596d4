"""CPU oracle for one AgentSAM speculative-decoding step.

TEST INFRASTRUCTURE ONLY.  These are plain, slow, obviously-correct CPU
implementations of what the hot path computes; they exist so the HIP library
can be checked element by element.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product path never
does, and this package never imports the product package.  The two share no
code.

  draft      - brute-force backward scan for the longest matched suffix and its
               continuation (C, see draft_oracle.c)          [Sec. 5.4.2, Alg. 4]
  attention  - fp64 softmax attention of the 1+k verification rows over a
               paged KV cache                                [Alg. 4 "Validate with main LLM"]
  accept     - first-index argmax per row and the matched draft prefix
                                                             [Alg. 4 "commit matched prefix"]
  sched      - AgentSched shadow price, scores and pick; the adaptive
               speculation switch and the depth / thresholds
               it is fed with                                [Alg. 3; Alg. 4 step 4]

Every function is pinned by tests that run without a GPU (worked examples,
closed forms, invariants, an independent brute force, library special cases),
with one exception: the choice among several weighted memories in
merged_draft_oracle follows a rule of this build (the paper names the merge
and its weights but prints no rule), so that rule is "parity unpinned"; the
per-memory drafts it chooses among are draft_oracle's and pinned as above.
"""
from .draft import (  # noqa: F401
    draft_oracle, draft_oracle_batch, build_oracle_lib, merged_draft_oracle, carried_match_len_oracle, draft_step_oracle,
)
from .attention import attention_oracle, attention_oracle_head          # noqa: F401
from .accept import accept_oracle                                        # noqa: F401
from .sched import (  # noqa: F401
    adaptive_k_oracle, agentsched_oracle, choose_k_oracle, expected_committed_oracle, switch_frontier_oracle,
)
