"""MI355X-native QR-Orth rotation-calibration step (DartQuant, arXiv 2511.04063).

``paper_2511_04063_amd.binding`` loads the HIP library (``libdartqr.so``) and exposes
its C entry points with the same names; ``paper_2511_04063_amd.synth`` draws the seeded
synthetic inputs.  Importing the package itself loads nothing native.
"""

__all__ = ["synth", "binding", "build"]
