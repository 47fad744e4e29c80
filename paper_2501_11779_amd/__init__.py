"""Tier-2 attention step of the two-tier offline-inference architecture, native on MI355X.

The product is the C-ABI library built from csrc/ (gh_kv_append, gh_decode_attention,
gh_decode_reduce); `binding` marshals torch device tensors into it and `workloads` draws the
seeded synthetic inputs.  There is no CPU fallback: the binding raises if the HIP library is
missing.
"""
__all__ = ["binding", "workloads"]
