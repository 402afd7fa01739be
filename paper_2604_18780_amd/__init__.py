"""MI355X-native streaming semi-CRF forward-backward (gfx950 HIP kernels behind a C ABI).

Importing the package is cheap and loads no native code: ``synth`` (input
generators) is plain numpy, and ``binding`` loads ``libsemicrf.so`` on first use
and raises if it is missing.
"""
__all__ = ["synth", "binding"]
