"""CPU oracle for one speculative-decoding step and the GammaTune controller.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 restatement of
what the GPU library computes.  It shares no code with the HIP path and is
imported only by the tests, by the smoke check and by the benchmark's CPU
baseline leg.  Nothing in the product package imports it.

Modules
-------
philox      Philox4x32-10 counter-based generator (Salmon et al., SC'11).
model       Llama-style decoder forward (RMSNorm, RoPE, MHA/GQA, SwiGLU).
sampling    softmax with temperature, index-order inverse CDF, the
            accept test u*q < p and the residual norm(max(0, p - q)).
spec        one speculative step (Background section: draft proposes gamma
            tokens, target verifies them in one pass) and the generate loop.
gammatune   the speculation-length controller (GammaTune section, eqs. for
            adaptive expansion and adaptive window estimation, Algorithm 1)
            and the GammaTune+ bookkeeping.

Parity pins (see tests/test_oracle_*.py): known-answer vectors for Philox,
closed forms and hand-worked trajectories for the controller, brute-force
enumeration of the accept/resample law on tiny vocabularies, hand-worked
values and flip tests for the decision margins, greedy speculative == greedy
target-only, a second forward built from torch CPU ops, structural
invariants (RoPE shift, GQA == MHA, cached == one-shot) and the cached pair
against one-shot forwards under roll-backs.

Parity unpinned by the paper (fixed by convention only, identical text on
both sides): hyper-parameter defaults (eta, delta, tau), which token an early
stop keeps, what the controller is fed after an early stop, the batch
extension, the Philox counter layout, and the synthetic confidence signal of
forced mode (its formula is this build's choice; its implementation here is
pinned by hand-worked values).
"""
