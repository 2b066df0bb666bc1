"""CPU oracles: one pipeline stage's forward pass, the pipeline's two ends, the 4-bit weight format, and the
models of the payload hand-off and of the pipeline's iteration time.  Test infrastructure only:
imported by tests/, by the smoke check and by the CPU-baseline leg of the
benchmark; never by the product package."""
from .stage_oracle import (  # noqa: F401
    OracleShape, rmsnorm, layernorm, gelu, rope_rotate, scaled_inv_freq, silu, slot_mapping, attention_rows,
    decoder_layer, stage_forward, new_pool,
)
from .ends_oracle import embed_tokens, last_rows, head_logits, greedy_tokens  # noqa: F401
from . import w4_oracle  # noqa: F401
from . import handoff_oracle  # noqa: F401
from . import pipeline_oracle  # noqa: F401
