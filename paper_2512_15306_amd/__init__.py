"""MI355X-native FP8 linear-layer path (absmax scaling, fused quantize+transpose, FP8 MFMA GEMMs).

``llmq``  -- Python binding of the C-ABI library (argument marshalling only; needs the built
             ``libllmq.so`` and a GPU, and raises if either is missing).
``synth`` -- seeded synthetic inputs of the benchmark configurations.
"""
__all__ = ["llmq", "synth"]
