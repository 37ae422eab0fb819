"""MI355X-native QA-LoRA adapted linear layer (gfx950 HIP kernels behind a C ABI).

``paper_2309_14717_amd.api`` is the thin Python binding of the C-ABI library;
``paper_2309_14717_amd.synth`` draws seeded synthetic inputs.  Importing the package
does not load the GPU library; the first call into ``api`` does, and fails loudly
when the library has not been built.
"""
__all__ = ["api", "synth"]
