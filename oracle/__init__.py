"""CPU oracle for the Ternary Weight Networks hot path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct CPU
statement of what the GPU library computes: a sort-based threshold ternarizer
(Eq. 3, Eq. 5, the rule of thumb of Sec. 2.3, Alg. 1 steps 4-7), direct-loop
convolution / inner product with the weights alpha*W~ (Eq. 2, Alg. 1 step 8) and
the straight-through backward (Alg. 1 steps 9-10).  It shares no code with the
HIP path and never imports it.  Only the tests, the smoke check and the
CPU-baseline leg of the benchmark may import it; the product never does.

Every function is pinned by tests that do not go through this package's own
formulas (hand-made vectors, closed forms, brute force, library routines);
nothing here is "parity unpinned".
"""

from . import ternarize, packing, conv  # noqa: F401
