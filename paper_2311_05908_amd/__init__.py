"""MI355X-native causal long FFT convolution (hand-written HIP behind a C ABI).

``paper_2311_05908_amd.fftconv`` is the Python binding of the C-ABI library;
``paper_2311_05908_amd.synth`` draws the seeded synthetic inputs.  Submodules
are imported on demand so that ``synth`` can be used without the HIP library.
"""
__all__ = ["fftconv", "synth", "build"]
