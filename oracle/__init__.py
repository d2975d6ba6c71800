"""CPU oracle for LoRANN's query phase.  TEST INFRASTRUCTURE ONLY.

Imported by `tests/`, by `__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`; never by the
library package.  `lorann_oracle.c` is the step-by-step query phase in plain C; `rrr_fit.py` is the
index-time reduced-rank-regression fit in numpy float64 used to pin the score model.
"""
