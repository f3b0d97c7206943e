"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package holds only input generation: tensor tables, access traces,
budgets and payload bytes.  None of the method's arithmetic (pool sizing,
placement, prefetch/evict decisions, stamping) lives here, so the oracle and
the library stay independent of each other while replaying identical inputs.
"""

from .traces import (  # noqa: F401
    R, W, RW, GROUP_16, GROUP_32, Workload, PHASE_FORWARD, PHASE_BACKWARD, PHASE_OPTIMIZER,
    config, config_names, gpt_shaped, llama_shaped, scaled_config,
    example_cpu_gpu, example_cpu_gpu_nvme, example_cpu_gpu_nvme_two_sizes, single_class_fwd_bwd,
    random_workload, optimizer_sweep, single_class_sweep, perturb_iteration, splitmix64,
)
from .payload import payload_bytes, payload_words, gaussian_fp16_bytes, workload_payload, PAYLOAD_SEED  # noqa: F401
