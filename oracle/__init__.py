"""CPU oracle for the PPO agent/trainer step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct numpy code that the tests, the smoke check and the benchmark's
``cpu_baseline`` leg compare the HIP path against.  Nothing in the product package imports it and
it imports nothing from the product package.

What it follows
---------------
* Structure (who does what, in which order): the paper's role descriptions (Section 3:
  environment simulator, agent, trainer) and the two sequential stages of synchronized training
  (Section 5.1: experience collection over a fixed number of agent-environment interactions, then
  model training on the collected batch); policy shapes follow Table 6.
* Numerics: the paper names PPO but prints none of its formulas, so each function follows the
  public definition it cites in its docstring (PPO clipped surrogate, GAE(gamma, lambda), Adam,
  Philox4x32-10, Box-Muller).

Every function here is pinned by ``tests/test_oracle_*.py`` against closed forms, brute force,
finite differences or an independent library, except where its docstring says "parity unpinned".
"""
from . import philox, ppo  # noqa: F401
