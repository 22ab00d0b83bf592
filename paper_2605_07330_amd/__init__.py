"""MI355X-native hot path of lossless sparse weight synchronisation (extract / apply).

``paper_2605_07330_amd.srs``   -- ctypes binding of the C-ABI library ``libsrs.so`` (HIP, gfx950).
``paper_2605_07330_amd.synth`` -- seeded synthetic workloads (inputs only).

Nothing is imported eagerly: ``synth`` is usable without the GPU library, and ``srs`` raises
at import when ``libsrs.so`` has not been built.
"""
__all__ = ["srs", "synth"]
