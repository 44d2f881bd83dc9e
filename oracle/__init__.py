"""Float64 CPU oracle for SAMA's meta-gradient step ("Making Scalable Meta Learning Practical").

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition the HIP path is checked
against.  It shares no code with the HIP library or its Python binding and must never be
imported by them; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.

Pins (tests/test_oracle_*.py; every function of the package has one):
  optim.adam_update          two textbook steps by hand
  optim.adam_adaptation      central difference of the Adam update u(g), the exact form of the
                             dropped eps term, first-step degeneracy                  (App. C)
  optim, reweight            weight decay as an L2 term, scheduled rates: SGD steps by hand,
                             the adaptation against a central difference        (App. B tables)
  sama_core.*                quadratic base losses with closed-form hypergradients,
                             biased regression closed forms                      (Eq. 5, App. D)
  sama_core + reweight       brute-force dense Hessian / mixed partial, exact IFT (Eq. 1-3)
  models.*, wnet.*           a second implementation from torch library layers with autograd
                             (also at the GPU's shape S = 128, head width 64, and with
                             key_padding_mask for padded batches), explicit loops
  corrector, reweight        soft-target cross-entropy special cases, torch autograd, differences
                             of the scalar base loss, dominant-prior limit            (Sec. 4.1)
  auxtask                    masked-token head against torch autograd, base gradient and
                             lambda-gradient against differences of the scalar base loss (Sec. 4.3)
  SGD invariant              adaptation reduces to a scalar step size           (Sec. 3.1-3.2)
  optim.sgd_momentum_update  heavy-ball steps by hand, du/dg by a central difference, the assembled
                             trajectory against hand-written steps          (App. B tables, reading)
  conditioning of Eq. 4      closed form of the adaptation for entries whose last gradient vanishes
                             and its peak at c2 sqrt(v') = eps_A; sensitivity of v to gradient noise
                             in the first steps of a run                                   (App. C)
The pins run at small shapes; the same code then runs the full-size workloads 3-5, for which
no second reference exists.
"""
