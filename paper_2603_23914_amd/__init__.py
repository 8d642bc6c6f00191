"""AttentionPack decode hot path for MI355X (gfx950): Python binding of the
C-ABI library `libattnpack.so` (hand-written HIP kernels).

`paper_2603_23914_amd.binding` marshals torch device pointers into the C calls
ap_compact / ap_select_ranks / ap_decode_attn; `workloads` holds the seeded
synthetic input generators.  There is no CPU fallback: importing `binding`
fails loudly when the shared library has not been built.
"""
__all__ = ["binding", "workloads"]
