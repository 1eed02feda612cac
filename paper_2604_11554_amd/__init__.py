"""MI355X-native rollout decoding (hand-written HIP for gfx950 behind a C ABI).

`binding` mirrors include/relax_rollout.h one to one; `engine` is the host-side
rollout loop (memory and integer bookkeeping only).  The HIP library must be
built first (`python -m paper_2604_11554_amd.build`); there is no fallback path.
"""
from . import binding
from .engine import Completion, Request, RolloutEngine, RolloutModel, StepOutput, StreamingRollout

__all__ = ["binding", "Completion", "Request", "RolloutEngine", "RolloutModel", "StepOutput", "StreamingRollout"]
