"""CPU oracle for the batched speculative-decoding verify step -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy statement of what the hot path computes: the decoder forward pass over
the draft rows of every branch (Section 3.1: the target model scores all draft positions of a sequence in one pass)
and the speculative-sampling accept / resample rule (Section 3.1; Algorithm 1, verification process).
It shares no code with the HIP library and is imported only by the tests, by the smoke check and by
the benchmark's CPU-baseline leg.  The product path never routes through it.

Pins (see tests/test_oracle_*.py): an independent library implementation of the same decoder
architecture, closed-form acceptance probabilities, exact enumeration on tiny vocabularies, the
chi-square losslessness test, closed forms of the temperature softmax, and structural invariants (branch
independence, relative-position invariance of rotary attention); for the rounds of Algorithm 1
(specdecode.py): with the draft model equal to the target every draft is accepted and the output must be
plain autoregressive sampling; a run with rejections equals, round by round, a cache-less recomputation from
the full token sequence; its first tokens follow the target's exact autoregressive law (chi-square on a tiny
vocabulary); the committed cache lengths equal the validated tokens of that replay minus the pending one.
The paper prints no worked numeric example, so absolute logit values are "parity unpinned" by the paper
itself; they are pinned by the library implementation.
"""
from .transformer import decode_rows, verify_forward, rms_norm, rope_rotate  # noqa: F401
from .specsample import (softmax_temperature, accept_resample, fixed_point_draw,  # noqa: F401
                         sample_from_probs, commit_lengths)
from .specdecode import speculative_rounds  # noqa: F401
from .spectree import (tree_from_k_config, tree_forward, accept_resample_tree, commit_rows_tree,  # noqa: F401
                       children_of, path_to)
