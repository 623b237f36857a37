"""CPU oracle of the multi-LoRA batched linear layer (fp64, plain loops).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does, and
this package imports nothing from the HIP path.
"""
from .reference import build_oracle, oracle_linear, oracle_workload, oracle_threads
from .plan_reference import plan_reference

__all__ = ["build_oracle", "oracle_linear", "oracle_workload", "oracle_threads", "plan_reference"]
