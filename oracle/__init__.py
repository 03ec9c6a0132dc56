"""CPU oracle for branch-isolated attention (ASPD, arXiv 2508.08895, Sec. 3.2-3.3).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this: it is
called by the tests, by the smoke check and by the benchmark's cpu_baseline leg.
It shares no code, table or helper with the GPU library and imports nothing
from it.

  token_table.py  the sequence as a list of token records, grown by replaying the
                  append history; position ids (Eq. 4); cache slots; the dense
                  mask (Eq. 2-3).
  attention.py    Eq. 1 in float64 with the explicit dense mask.
  attention_ref.c the same in plain C loops with OpenMP and no BLAS (attention_c.py loads it): a second
                  writing that the pins also run against, and the one bench.py times on the host's cores.
  rope.py         rotary encoding of the new tokens by their Eq. 4 position ids and their
                  placement in the cache (the step between the metadata and the attention call).

Pins (tests/test_oracle_*.py): hand-derived worked example, brute-force visible
sets, closed-form counts and positions, uniform-weight means, single-key and
equal-value cases, a library attention routine for the one-branch case, branch
isolation, branch permutation, merge == unmasked attention over gathered rows;
mixed batches: hand-derived two-sequence example, equality with sequences decoded alone;
rotary encoding: hand-derived example, complex multiplication, shift invariance of scores.
Parity unpinned: agreement of Eq. 1-4 with a trained model's behaviour (needs
weights and datasets, out of scope).
"""
from .token_table import TokenTable, StepMeta, MAIN  # noqa: F401
from .attention import attend, attend_queries  # noqa: F401
from .rope import rotate, rope_append  # noqa: F401
