"""CPU oracle for the asynchronous Local-SGD hot path (test infrastructure only).

Plain, slow, obviously-correct numpy code written from the paper: the decoder-LM loss and
its hand-derived gradient, AdamW as the inner optimiser, the pseudo-gradient, the Delayed
Nesterov (DN) outer update (Alg. 3), Dynamic Local Updates (Eq. DyLU) and the asynchronous
task scheduling loop (Alg. 2 with its get_worker() helper) on a simulated clock.

Nothing in the product path may import this package: only tests/, the smoke check in
__graft_entry__.py and the cpu_baseline leg of bench.py use it.  It shares no code with
the HIP library; both are fed the same seeded arrays from ``als_inputs``.

Every function works in the dtype of the arrays it is given: float64 for gradient checks
and pins, float32 for parity runs and timing.

Parity status: every function here is pinned by tests/test_oracle_*.py against closed
forms, paper-printed identities, library routines or finite differences.  The whole
multi-round run has no paper-printed trajectory to compare with (the paper's numbers are
perplexities on a corpus and checkpoints that are not available): it is pinned only through
the composition of those pins and the synchronous special case -- "parity unpinned" beyond
that.
"""
