"""MI355X-native sparse-embedding path (dedup + dynamic hash table lookup + sparse Adagrad).

``binding`` mirrors the C ABI of ``include/mtgr_emb.h`` one to one; ``table`` owns the torch
tensors that serve as device memory.  The compute is in ``libmtgr_emb.so`` (hand-written HIP for
gfx950); importing this package without the built library raises.
"""
from . import binding  # noqa: F401
from .binding import F32, BF16, EmbError, load  # noqa: F401
from .table import EmbeddingTable, StepBuffers, forward, forward_two_call, backward, forward_fused, backward_fused  # noqa: F401

load()
