"""MI355X-native denoising step and cache-hit resume loop of a latent video
diffusion transformer, behind a C-ABI library.  `synth` (seeded inputs) imports
without the native library; everything else needs it built."""


def __getattr__(name):
    # the binding loads the native library on first use, and raises if it is missing
    if name == "synth":
        import importlib
        return importlib.import_module(".synth", __name__)
    from . import binding
    return getattr(binding, name)
