"""CPU oracle for the sparse fully-connected training step of Mixed Sparsity Training.

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow, obviously-correct
statement of what the hot path computes, written from the paper (Sec. 3.1
"Sparsity Variation", Sec. 3.2 / Algorithm 1 "Topology Evolution by MG",
Sec. 3.3 strided attention pattern, App. "FLOP Calculation").  Only the test-suite, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it; the product (the HIP library and
its Python binding) never does and shares no code with it.

All floating-point work is done in float64 with numpy; nothing here is blocked,
fused or reordered beyond what the definitions state.

Pin status (see tests/test_oracle_*.py):
  schedule.density / schedule.zeta  pinned: closed-form end points, hand-computed
                                    stage values with the paper's hyper-parameters,
                                    step-average, monotonicity.  The choice that the
                                    first stage change happens at t = Delta_W (not
                                    t = 0) is a reading, not pinned by the paper.
  products.*                        pinned: pure-Python loop brute force, density-1
                                    reduction to a plain matrix product, adjoint
                                    identities, linearity.
  mixed_growing.counts              pinned: conservation invariant, worked numbers
                                    for the 768->3072 layer, clamp cases.
  mixed_growing.randk_key           pinned: the published SplitMix64 test vector.
  mixed_growing.update              pinned: brute force with Python's sorted() on tiny
                                    inputs, set invariants, R=0 / R=1 special cases,
                                    chi-square uniformity of the random part; the
                                    lambda prune criterion by brute force on dyadic
                                    values, lambda = 0 and lambda -> large.
  allocation.erdos_renyi_density    pinned: hand-computed densities of the GPT-2-small block
                                    and of a saturating pair, budget conservation, an
                                    independent bisection solve, special cases.
  flops.fc_forward / transformer    pinned: the FLOPs column of the main results table
                                    (static-sparse 80 %, Tiny, dense), multiply-add brute
                                    counts.  The table's MST row (219.4 G) is not
                                    reproduced by any reading tried (226.2 G here): the
                                    schedule average is parity unpinned against it.
  attention_mask.strided_mask       pinned: the printed Q_atten of strides 128 and 256,
                                    the set definition, a closed-form count.
"""
