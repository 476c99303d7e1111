"""Seeded synthetic inputs for the CachePrune KV-sharing path: prompts, masks,
free lists (``gen``) and KV values (``kvgen``).  Serves the CPU oracle and the
GPU library alike and contains none of the method's arithmetic."""
from . import gen, kvgen  # noqa: F401
