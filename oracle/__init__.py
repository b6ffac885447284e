"""CPU oracle (test infrastructure only; never imported by the product path)."""
from .binding import (build, monarch_forward, blast_forward, dense_forward,
                      materialize_monarch, materialize_blast, monarch_middle_perm,
                      lowrank_forward, materialize_lowrank, monarch_rect_forward,
                      OUT_INTERLEAVED, OUT_BLOCKED)
