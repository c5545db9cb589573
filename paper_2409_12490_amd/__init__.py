"""MI355X-native CritiPrefill prefill-attention path.

``binding`` marshals arguments into the C ABI of ``libcritiprefill.so`` (hand-written HIP kernels for
gfx950); ``synth`` draws the seeded synthetic inputs; ``build`` compiles the library; ``studies`` holds
measurements beyond the headline benchmark.  Importing the package loads nothing.
"""
__all__ = ["binding", "synth", "build", "studies"]
