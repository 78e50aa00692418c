"""CPU oracle for one SwarmSGD interaction (arXiv 1910.12308).

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow reference that the
HIP library is checked against.  It shares no code with the HIP path and must
never be imported by the product package: only the tests, the smoke entry
point and the benchmark's CPU-baseline leg may use it.

Everything here follows the paper's Algorithm 1, its Section 3 prose
("Parallel Execution", "The Communication Procedure") and Corollary 2.1
(the quantizer's three properties).  Floating point is float64 except where a
float decides an integer (the stochastic-rounding decision and the decoding
key), which is done in float32 with single IEEE operations so that both sides
take the same decision.

Pin status per function (what each is checked against, other than itself):
  philox4x32_10            rocRAND's Philox4x32-10 host-callable engine, compiled
                           at test time from the vendor header (library routine)
  stochastic_round         closed-form up-probability, exhaustive over all 2^16
                           random halves; unbiasedness on averaged trials
  code / decode            brute force over integers for every b
  pack / unpack            round trip + explicit byte images
  gossip_round (bits=0)    swarm mean preserved; potential drop = |Xi-Xj|^2/2
                           (appendix, proof of the per-step potential bound)
  gossip_round (quantized) both members of a pair hold the same average when
                           both decodes succeed; contraction on the complete
                           graph by enumeration
  interact (Algorithm 1)   responder receives the plain average; snapshot rule; exact
                           potential identity of the per-step lemma; wrapped value under
                           decode failure
  local steps, diagonal    closed form w_H = c + (1-eta a)^H (w_0 - c) at sigma=0; with noise,
                           mean and variance of w_H against the closed form of the linear recursion
  noise_normals            one generator call written out by hand; scipy's normal law
                           (Kolmogorov-Smirnov), moments, independence inside and across calls
  local steps, least sq.   numpy gradient A^T(Ax-b) on the same batch
  local steps, MLP         torch.autograd in float64 on the same batch
  sample_pair              every ordered edge (i, j) equally likely per 1/(n deg i), chi^2
  sample_matching          validity + brute-force greedy on tiny graphs + chi^2
  sample_stale             uniform on {0..S}, limited to the rounds that exist
  steps_of (geometric H)   E[H_i] = H and E[H_i^2] = 2H^2 - H (appendix, local steps)
  pair_scale               smallest power of two inside the decoding radius; no decode fails
  scale "global_linf"      update rule recomputed from the published codes in plain Python;
                           equals the fixed-scale rule while the scale stands still; recovers
                           from a wrong starting scale; stale read across a scale change by hand
  apply_mode "inplace"     X_i' = (w_i + w_j)/2 with w the closed-form local-step result
  potential                definition, and the Laplacian inequality of the appendix
  potential_hat            three nodes by hand; Gamma-hat <= 2A + 2B of the appendix along a run,
                           with the models and means at each node's last initiation tracked apart
  lattice_coordinate       clamp values; what is not a number is flagged and saturates
  whole trajectories       parity unpinned beyond the invariants above
"""
