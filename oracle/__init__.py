"""CPU oracle for the VARCO layer hot path — TEST INFRASTRUCTURE, not product code.

Plain numpy in fp64, written from the paper (Sections II-IV, Definition 1, Algorithm 1, Appendix
"Compression Mechanism" / "Scheduler"). It shares no code with the HIP library and must never be
imported by it: only tests, the smoke check and the benchmark's CPU-baseline leg may use it.

Modules
    mask       keyed choice of the kept feature positions, kept-count rule, ratio schedulers
    partition  per-partition CSR / halo / boundary index structures from a global graph
    layer      compress, decompress, one partition's layer forward and backward, whole-network step

Pins (tests/, `-m "not gpu"`): dense-adjacency brute force of eq. (2) at ratio 1 and of the global-mask
formula at any ratio, partition-count invariance, central finite differences, adjoint identities,
compressed sizes, mask statistics against the closed-form error moment of Definition 1.

Parity unpinned: the *particular* index values the keyed generator yields (the paper fixes only that a
key shared a priori lets the decoder recover the positions); they are fixed by this repository's written
mask rule, implemented here and, independently, in the HIP library.
"""
