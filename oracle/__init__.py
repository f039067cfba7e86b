"""CPU oracle for the ragged-cache attention path -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this directory.  It may be used by the
tests, by the smoke check and by the benchmark's ``cpu_baseline`` leg, and by
nothing else.  It shares no code with the HIP library: the only thing both sides
see are the seeded input tensors.

Parts (each cites the passage of the paper it follows):

* ``oracle.policy``    -- which history frames a head keeps and attends to
                          (Sec. 2.2; Sec. 4.2 Eq. 4, Eq. 5, shared sink/recent).
* ``oracle.pool``      -- the per-head ragged KV pool as a list of frames
                          (Sec. 2.2 write-back; Sec. 4.3 flattened layout).
* ``oracle.attention`` -- softmax attention of every head over its own frames
                          (Sec. 2.1 Eq. 1, Sec. 2.2 Eq. 2, Sec. 4.3), C with
                          double accumulation.

Parity status: every function here is pinned by ``tests/test_oracle_*.py``
against hand-worked fixtures, closed forms, brute force on tiny inputs or a
library routine.  The paper prints no worked numeric example of an attention
output or of a frame list, so nothing here is pinned against the authors' own
implementation.
"""
