"""fp64 CPU oracle for KDA -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the CPU-baseline leg of the bench may import
this package.  It never imports the HIP package and shares no code with it.

`kda_forward` / `kda_step` / `kda_steps_pooled` call the plain C recurrence in ``kda_oracle.c``
(paper Section 3, Eq. (1)); `chunkwise_ref.kda_chunkwise` is a second, numpy
fp64 statement of the same function written from the chunkwise equations of
Section 3.1, used to pin the recurrence (chunk-size invariance).
"""
from .recurrence import build, kda_forward, kda_step, kda_steps_pooled, num_threads  # noqa: F401
