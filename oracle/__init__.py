"""CPU oracle for DSSP parameter-server training.

TEST INFRASTRUCTURE ONLY.  Everything under this directory is a plain, slow,
obviously-correct CPU restatement of what the paper's method computes.  It is
imported by the tests, by the smoke check and by the benchmark's CPU-baseline
leg, and by nothing else; it shares no code with the HIP library and never
imports it.

  dssp_rules.py  integer event simulator + BSP / ASP / SSP / DSSP decision
                 rules (Alg. 1 server part, Alg. 2 synchronization controller)
  nn_layers.c    fp64 layer forward / backward as direct loops (OpenMP)
  nn.py          ctypes wrappers + the three networks, gradient = mean over
                 the mini-batch of per-sample loss gradients (Alg. 1, worker
                 step 4)
  ps.py          whole emulation: simulator + numerics (pull, gradient, apply)
"""
