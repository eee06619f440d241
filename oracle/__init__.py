"""CPU oracle for the Hop decentralized-update hot path (arXiv 1902.01064).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, sequential statement
of what the path computes, written from the paper: a discrete-event run of the
queue protocol (Sections 4.1-4.4, 5, 6.1, 6.2), the iteration-weighted reduce
(Eq. 2), the standard decentralized update (Figure 1 "Standard Decentralized
Training") and a hinge-loss linear SVM minibatch subgradient.  It shares no code
with the HIP library and never imports it.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it; the product never does.

Modules
  rng       counter-based random numbers the method draws (delays, minibatches,
            synthetic gradients)
  protocol  event-driven run of the protocol -> list of STEP / JUMP records
  arith     weights (Eq. 2 x mixing weights), SVM subgradient, reduce + apply
  waves     level schedule of records over ring slots + its validity check
  brute     exhaustive untimed enumeration of the protocol for tiny graphs
  brute_na  the same for NOTIFY-ACK (Section 3.3)

Parity pins (tests/test_oracle_*.py, tests/test_next_*.py): closed forms X_{k+1} = W^T X_k - eta G_k (parallel
approach) and X_{k+1} = W^T (X_k - eta G_k) (serial approach), matrix powers, eigenvalue contraction, Theorem 1 /
Theorem 2 bounds, the token identity, the iteration-gap table (NOTIFY-ACK row included), the paper's worked
examples, Eq. 2 by hand, numpy matmul gradient, finite differences, exhaustive enumeration.  Two readings the
paper gives no algorithm for - the hybrid accept rule (backup workers together with staleness) and the skip
trigger / size - are pinned by traces worked by hand under those readings (tests/golden/hybrid_trace.txt,
jump_trace.txt); they remain readings, stated in the repository's design notes.
"""