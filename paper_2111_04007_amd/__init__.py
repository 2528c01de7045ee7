"""MI355X-native pipeline-stage compute (forward / recompute / backward with
fp32 gradient accumulation) behind a C ABI; see include/varuna_stage.h."""
from .synth import CONFIGS, StageConfig  # noqa: F401
