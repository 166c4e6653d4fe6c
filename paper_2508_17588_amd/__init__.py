"""MI355X-native cached DiT denoising step (HERO): HIP kernels behind a C ABI.

`binding` mirrors the entry points of include/hero.h one to one; `build` compiles
libhero.so for gfx950.  There is no CPU or PyTorch fallback path.
"""
from . import binding  # noqa: F401
from .binding import HeroCache, HeroError, load_library, make_config  # noqa: F401
