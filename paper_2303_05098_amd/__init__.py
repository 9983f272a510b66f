"""MI355X-native SpMV format engine and format auto-tuner (six storage formats,
CSR-to-format conversions, sparsity-pattern features, run-first and tree tuners).

Importing this package loads nothing heavy.  ``paper_2303_05098_amd.mo`` is the
binding over the C-ABI library (HIP kernels); ``paper_2303_05098_amd.synth``
holds the seeded input generators; ``paper_2303_05098_amd.fit`` the host-side
tree trainer used by the tuner sweep.
"""
__all__ = ["mo", "synth", "fit", "build"]
