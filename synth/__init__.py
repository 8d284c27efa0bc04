"""Seeded synthetic inputs (shapes, weights, prompts, masks) shared by the oracle and the
HIP path.  Holds no arithmetic of the method itself."""
from .generators import (ModelDesc, CONFIGS, WORKLOADS, make_weights, make_router,
                         make_prompt, make_skip_mask, make_interval_mask, torch_dtype)

__all__ = ["ModelDesc", "CONFIGS", "WORKLOADS", "make_weights", "make_router",
           "make_prompt", "make_skip_mask", "make_interval_mask", "torch_dtype"]
