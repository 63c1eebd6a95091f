"""CPU oracle: a plain, slow, float64 NumPy statement of what the hot path computes.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this package:
it is used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline
leg.  It shares no code with the HIP library and never calls it.

Modules (each function cites the passage of the paper it follows):
  dnn        forward / cross-entropy backward / SGD update of the sigmoid-softmax DNN
  averaging  parameter averaging across replicas and the local-SGD driver loop
  philox     Philox4x32-10 counter-based generator and the uniform it yields
  rbm        one CD-1 minibatch update (Gaussian or Bernoulli visible units)
  ngsgd      online low-rank natural-gradient preconditioner

Pins (tests/test_oracle_*.py, run without a GPU): finite differences, softmax
identities, closed-form logistic regression, the averaging/gradient-averaging
identity of Sec. 3, brute-force CD-1 expectation on a 4x3 RBM, Philox known
answers, dense-matrix checks of the NG-SGD algebra, hand-worked examples of its
floors and a dense replay of its first call.  That the NG-SGD constants,
initial state and number of initial folds are those of the cited algorithm
(the paper itself does not print them): parity unpinned.
"""
