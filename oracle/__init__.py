"""CPU oracle for the per-rank matrix-optimizer step of Canzona (arxiv 2602.06079).

THIS PACKAGE IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow,
fp64 numpy implementation of what the device library computes, written from
the paper so that a reader can check it against the paper by eye.  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import it.
It shares no code with the HIP/C++ library and never imports it.

Modules
-------
partition   Algorithm 1 (alpha-balanced greedy LPT partitioning, Sec. 3.2 and
            the walkthrough in App. C) plus the load-balance diagnostics of
            Eq. 2, Eq. 3 and Eq. 6.
microgroup  Same-shape batching of one rank's matrices (the deterministic
            (cost, id) ordering of Algorithm 2, Phase 1, applied to shape
            classes, with a capacity cap in the spirit of C_max).
tp_schedule TP micro-group construction with greedy rollback and the min-heap LPT solver
            (Algorithm 2; Algorithms 3 and 4 in App. C).
shampoo     The Shampoo operator the paper runs through the same planner (App. C,
            "Generalization to Other Optimizers"): Kronecker-factor statistics, inverse
            fourth roots by eigendecomposition, preconditioned update.
soap        The SOAP operator of the same experiment: Adam in the eigenbasis of those
            statistics, the basis refreshed by one round of orthogonal iteration (QR).
muon        The Muon operator named in Sec. 4.1 / App. B.3: momentum,
            Frobenius normalisation, k Newton-Schulz steps, scaled update;
            TP column-fragment gather/scatter of Sec. 4.1 stages (1) and (3).

Parity pins (tests/test_oracle_*.py): every function here is pinned to
something other than itself - SVD closed forms and the polar factor for the
Newton-Schulz iteration, a scalar-map grid for the quintic band, defining identities
and diagonal / rank-one / SVD closed forms for the Shampoo step, torch's Adam, the polar
factor and the defining properties of the QR refresh for the SOAP step, hand-worked
partitions, exact-rational replays, brute-force enumeration of cut vectors,
and structural invariants.  The paper's measured load-balance ratios depend on
a bucket layout it does not give; they are not pinned.
"""
