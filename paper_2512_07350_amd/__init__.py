"""MI355X-native hot path of Latent Parallelism: partition, attention, reconstruct.

``paper_2512_07350_amd.binding`` wraps the C-ABI library (built from ``csrc/``);
``paper_2512_07350_amd.synth`` holds the seeded synthetic inputs.  Nothing is
loaded at import time; the library is opened on first use and its absence is an
error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
