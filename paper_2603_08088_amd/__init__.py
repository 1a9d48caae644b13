"""MI355X-native teacher verification step of tree speculative decoding.

The five operations of the step (tree-mask construction, tree-masked attention
against prefix + tree KV, sentinel-free path gather, greedy posterior
acceptance, commit of the accepted path's KV) are hand-written HIP kernels for
gfx950 behind a C ABI (``include/eagletv.h``).  ``api`` is the thin Python
binding (argument marshalling only); ``synth`` holds the seeded synthetic
workload generators, which contain none of the method's arithmetic.

Importing this package does not load the HIP library; ``api`` loads it on first
use and raises if it has not been built.
"""

__all__ = ["api", "synth", "build"]
