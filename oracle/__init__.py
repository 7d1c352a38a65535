"""CPU oracle (test infrastructure only): kvl_oracle.c defines the data movement,
sched_oracle.py the scheduling rules and the P/D range."""
from .kvl_oracle import (  # noqa: F401
    build, payload_bytes, total_hit_tokens, check, pack, unpack, stream_layers,
    pack_range, unpack_range, check_range_scatter,
    fullblock_bytes, fullblock_count, fullblocks_to_pool, pool_to_fullblocks, stream_layers_fullblocks,
    OK, E_ARG, E_TABLE, E_BLOCK, E_DUP,
)
