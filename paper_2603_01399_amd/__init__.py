"""MI355X-native int8 weight-streaming verification kernels (C-ABI library + thin binding).

``from paper_2603_01399_amd import binding`` loads the HIP shared library; there is
no CPU fallback: a missing library raises.
"""
__all__ = ["binding", "synth"]
