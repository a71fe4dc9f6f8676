"""Plain CPU oracle of the denoising path (test infrastructure, not product code)."""
from . import cache, dit, sampler  # noqa: F401
