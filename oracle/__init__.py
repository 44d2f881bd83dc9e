"""Float64 CPU oracle for SAMA's meta-gradient step ("Making Scalable Meta Learning Practical").

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition the HIP path is checked
against.  It shares no code with the HIP library or its Python binding and must never be
imported by them; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.

Pins (tests/test_oracle_*.py):
  optim.adam_adaptation      central difference of the Adam update u(g)           (App. C)
  sama_core.*                quadratic base losses with closed-form hypergradients,
                             biased regression closed forms                      (Eq. 5, App. D)
  sama_core + reweight       brute-force dense Hessian / mixed partial, exact IFT (Eq. 2)
  models.*, wnet.*           central differences of their own float64 forward
  SGD invariant              adaptation reduces to a scalar step size           (Sec. 3.1-3.2)
Parity unpinned: the full-size encoder numerics of workloads 3-5 have no reference outside
this oracle beyond the gradient checks above on small shapes.
"""
