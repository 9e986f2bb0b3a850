"""MI355X-native trial evaluation and search loop of OpEvo (arxiv 2006.05664).

`binding` holds one Python function per entry point of the C-ABI library `libopevo.so`
(declared in include/opevo.h); `synth` generates the seeded synthetic workloads.
Importing the package loads the library and fails loudly if it has not been built.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
