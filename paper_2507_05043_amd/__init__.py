"""MI355X-native forward pass of one pipeline stage (decoder layers over a mixed prefill/decode
micro-batch with a paged KV cache): hand-written gfx950 kernels behind a C ABI, with a thin
ctypes binding.  `synth` draws the seeded synthetic inputs."""
from . import synth  # noqa: F401
from .stage import (  # noqa: F401
    Stage, StageError, StageConfig, StageLayerWeights, StageTaps, KERNEL_CLASSES, load_library,
    stage_check_batch, stage_kv_element_offset, stage_kv_layer_bytes, stage_workspace_bytes,
    stage_kernel_name,
)
