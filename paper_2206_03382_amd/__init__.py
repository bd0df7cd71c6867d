"""MI355X-native hot path of a Tutel-style MoE layer: gate top-k + slot assignment, sparse encode/decode, expert FFN.

The HIP library is loaded lazily by `paper_2206_03382_amd.moe`; importing the package (or `synth`) needs no GPU.
"""
__all__ = ["synth", "moe"]
