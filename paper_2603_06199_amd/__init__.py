"""MI355X-native FlashPrefill prefill-attention path (gfx950 HIP kernels behind a C ABI).

``paper_2603_06199_amd.binding`` is the thin ctypes layer over ``libflashprefill.so``;
``paper_2603_06199_amd.synth`` draws the seeded synthetic inputs.  Nothing here falls back to a
CPU or PyTorch implementation: without the built library the binding raises.
"""
__all__ = ["binding", "synth", "build"]
