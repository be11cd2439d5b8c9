"""CPU oracle for the batched speculative verify step (test infrastructure).

Plain, slow numpy fp64 code written from the paper's definitions.  It is used
by the tests, by the smoke check and by the benchmark's CPU-baseline leg only;
the product path never imports it, and it shares no code with the HIP library.

Parity pins (see tests/test_oracle_*.py): every function below is pinned by
closed forms, brute force on tiny inputs or the method's defining invariant,
except the *acceptance rates* the paper reports in Table 1, which need trained
weights and datasets that are not available: those are "parity unpinned".
"""
from .model import Model, KVCache                                   # noqa: F401
from .drafts import (context_ngram_groups, context_rows, bigram_scores, rank_ids,   # noqa: F401
                     Bigram, ModelBigram, unigram_distances, UnigramDrafts, build_drafts)
from .verify import (accept_lengths, select_winner, State, prefill, verify_step,    # noqa: F401
                     commit, greedy_plain, greedy_plain_cached, greedy_speculative, adaptive_context_cap)
