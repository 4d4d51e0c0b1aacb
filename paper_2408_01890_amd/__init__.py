"""LiSA attention layer (cross-layer attention sharing) for AMD MI355X.

`paper_2408_01890_amd.lisa` is the thin binding of the C-ABI HIP library
(`lisa_attn_prefill`, `lisa_attn_decode`, `std_attn_scores`); `paper_2408_01890_amd.synth`
draws the seeded synthetic workloads.  Importing the package loads neither.
"""
__all__ = ["lisa", "synth"]
