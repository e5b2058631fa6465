"""CPU oracle for the pipeline-stage compute (forward + backward of a run of
decoder layers on one tensor-parallel shard, with gradient accumulation).

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain numpy implementation of
the textbook definition of the layers, kept deliberately simple so it can be
checked by eye.  Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does, and this
package never imports the HIP path.

Pins (tests/test_oracle_*.py): central finite differences in float64 for every
backward formula, an independent autograd re-statement of the layer, softmax
row sums, bit-exact causality, K-microbatch accumulation against the
concatenated batch, tensor-parallel partial sums against the unsharded block,
closed-form special cases (S = 1, equal scores, RoPE relative-position
property, zero second matrix), and the paper's worked example of the
column / row split (Section II-B).

Unpinned: nothing in this package is unpinned.  (The profile *times* of the
product are measurements and have no oracle; its byte counts are checked
against integer identities in the tests.)
"""
from .stage_ref import *  # noqa: F401,F403
from . import cost_ref  # noqa: F401
