"""The GPU tests reach the workload runner of the package under its old local name."""
from paper_2509_09682_amd.runner import (  # noqa: F401
    device_sampler, run_hip, run_hip_sampled, sample_hip, to_device,
)
