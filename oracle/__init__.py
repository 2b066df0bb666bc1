"""CPU oracle of one pipeline stage's forward pass.  Test infrastructure only:
imported by tests/, by the smoke check and by the CPU-baseline leg of the
benchmark; never by the product package."""
from .stage_oracle import (  # noqa: F401
    OracleShape, rmsnorm, rope_rotate, silu, slot_mapping, attention_rows,
    decoder_layer, stage_forward, new_pool,
)
