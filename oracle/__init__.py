"""Float64 CPU oracle for one worker's NG-SGD minibatch step.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
NumPy float64 statement of what the paper's online natural-gradient SGD step
computes.  It exists to check the HIP implementation; it shares no code with
it and must never be imported by the product path.  Only the test-suite, the
smoke check and the benchmark's CPU-baseline leg may import it.

Modules
  online_ng            online preconditioner, definitional form (App. B.1-B.2,
                       B.3.1, B.3.2): explicit R_t, D_t, rho_t.
  online_ng_efficient  the same update in the efficient form of App. B.3 / B.5
                       (W_t, H, J, K, L, Z, A_t, B_t) - used by the tests to pin
                       the formulas against the definitional form.
  simple_ng            the simple method (App. A): hold-one-out Fisher factors
                       from the current minibatch, definitional and efficient forms.
  network              forward / objective / backward / precondition / update
                       (Sec. 2, Sec. 4.5-4.6).
  averaging            parameter averaging across replicas (Sec. 3.1).

Parity pins: every function here is pinned by tests/test_oracle_*.py against
brute-force dense algebra, closed forms and invariants fixed by the paper.
Parity unpinned: trajectories on the paper's speech data (data not available).
"""
