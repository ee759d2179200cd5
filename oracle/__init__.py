"""CPU oracle of the TS-DP speculative denoising round.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the hot path computes: DDPM
schedule tables, the Philox4x32-10 noise stream, the denoiser forward, the
drafter rollout, the batched verification and the likelihood-ratio acceptance
with reflection-maximal coupling.  It shares no code with the HIP library and
must never be imported by the product package: only tests, the smoke check and
the benchmark's cpu_baseline leg may use it.

Pins (see tests/test_oracle_*.py): schedule closed forms, Philox known-answer
vectors, Gaussian log-density ratio, acceptance probability 2*Phi(-|d|/2),
reflection isometry and marginal law, identity-drafter invariant, whole-chain
law against the closed-form linear-Gaussian chain, transformer blocks against
torch CPU library routines.  The absolute output of a full round on random
weights has no external reference ("parity unpinned" beyond the composition of
the pinned parts).
"""
