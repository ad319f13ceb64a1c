"""Seeded synthetic inputs for the CO2 outer-update path.

This module is shared by the oracle's tests and the HIP path's tests/bench.  It
holds segment tables (the per-tensor sizes of the model shapes the workloads
imitate), the hyper-parameters of the five workload configurations, and seeded
random fills.  It holds none of the method's arithmetic and imports neither the
oracle nor the HIP package.
"""
from .tables import (equal_table, gpt_table, llama_table, shard_of_table,  # noqa: F401
                     CONFIGS, WorkloadConfig, config_table)
from .draws import (seed_for, fill_normal_, fill_student_t_, fill_bf16_normal_)  # noqa: F401
