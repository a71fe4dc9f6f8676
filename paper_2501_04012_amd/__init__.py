"""MI355X-native denoising step and cache-hit resume loop of a latent video
diffusion transformer, behind a C-ABI library.  `synth` (seeded inputs) imports
without the native library; everything else needs it built."""
import importlib


def __getattr__(name):
    if name in ("synth", "binding", "build"):
        return importlib.import_module("." + name, __name__)
    # the binding loads the native library on first use, and raises if it is missing
    return getattr(importlib.import_module(".binding", __name__), name)
