"""Synthetic inputs shared by the CPU oracle's tests and the GPU library's
tests and benchmark.  No latency model, no scoring, no search lives here."""
from .traces import (Recipe, Trace, generate, regroup, recipe, config, random_trace, pack_bits,
                     unpack_bits, CONFIG_NAMES, KV_TOKEN_BYTES)
from .placements import (random_placements, edge_placements, random_moves, moves_to_records,
                         OP_SET, OP_SWAP, OP_SHIFT, MOVE_FIELDS)
