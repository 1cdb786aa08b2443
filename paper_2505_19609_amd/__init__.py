"""MI355X-native packed varlen causal attention (forward + backward) for one
scheduled micro-batch of whole short sequences and context-parallel query
shards of long ones.  The compute lives in ``csrc/`` (HIP, gfx950) behind the
C ABI declared in ``include/skrull_attn.h``; :mod:`.binding` only marshals
arguments.  Nothing here falls back to the CPU."""

__all__ = ["binding", "workloads"]
