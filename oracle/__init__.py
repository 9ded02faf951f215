"""CPU fp64 oracle for the normalized-Laplacian eigenproblem.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares no code with the HIP library and never imports it; the library
never imports this package.

Contents
--------
``laplacian``   degrees, D^-1/2 scaling, the operator S = D^-1/2 W D^-1/2, dense L = I - S
                (Section II Step 2 and Section IV-B, in the symmetric form).
``dense``       plain definition: dense symmetric eigendecomposition of L, first k pairs.
``lanczos``     single-vector Lanczos with full reorthogonalization (classical Gram-Schmidt
                applied twice), thick restart, locking and random re-injection
                (the restarted Lanczos of Section IV-B / Algorithm 3, made multiplicity-safe).
``components``  exact spectrum by connected components: closed-form null space
                D^1/2 1_C / sqrt(vol(C)) plus per-component eigenproblems.
``compare``     residuals, principal angles and containment defects used by the parity tests.

Every function is pinned by ``tests/test_oracle_*.py`` to closed forms (ring, path, complete,
complete bipartite, hypercube, disjoint unions), to invariants (spectrum in [0, 2], trace,
Frobenius norm, scaling and relabeling invariance, orthonormality) and to each other.
"""
