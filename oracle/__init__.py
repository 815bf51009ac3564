"""CPU fp64 oracle for one block-wise diffusion decode step (Streaming-dLLM).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import this package; only the tests, the smoke check and the
bench's cpu_baseline leg do.  The oracle shares no code with the HIP path: it is
the plain definition of each operation written out in numpy float64, with no
tiling, fusion or reordering, so that it can be checked against the paper by eye.

Every function is pinned by tests that do not re-use its own formula: scalar
brute force on tiny inputs, closed forms, invariants and library special cases
(see tests/test_oracle_*.py).  The paper prints no worked numeric example of a
decode step, so there are no paper-supplied golden values; tests/golden/ holds
closed-form values derived by hand from the paper's equations.
"""
from .attention import block_attention, compose_rows  # noqa: F401
from .unmask import confidence_unmask, dynamic_threshold, row_confidence  # noqa: F401
from .kv_append import kv_append  # noqa: F401
from .suffix import suffix_keep_indices  # noqa: F401
from .lm_head import lm_head_logits, lm_head_unmask  # noqa: F401
from .rope import pruned_positions, rope_gathered, rope_rotate  # noqa: F401
