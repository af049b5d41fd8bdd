"""AnchorAttention sparse causal prefill for MI355X (gfx950).

``paper_2505_23520_amd.api`` is the thin binding over the C-ABI library
(``libanchor_attention.so``, hand-written HIP); ``paper_2505_23520_amd.synth``
draws the seeded synthetic workloads.  Importing the package does not load
the GPU library; importing ``api`` does, and fails loudly if it is not built.
"""
__all__ = ["synth"]
