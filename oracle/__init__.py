"""Float64 CPU reference ("oracle") for the fine-tuning step.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark; never by the product package.
"""
from .pack import pack, PackError, ROLE_SYSTEM, ROLE_USER, ROLE_ASSISTANT, ROLE_TOOL  # noqa: F401
from .model import Config, forward, backward, train_step, merge_lora, config_from_shape  # noqa: F401
from .adamw import adamw_update, cosine_lr  # noqa: F401
