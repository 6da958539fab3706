"""MI355X-native rollout decode step (Qwen2-style GQA decoder over paged, ragged KV caches).

The package holds two things and nothing else:

* ``synth``   -- seeded synthetic workloads (model shapes, weights, KV fill, lengths, block
                 tables).  It contains none of the decode arithmetic and is the only module
                 shared by the HIP path and the CPU checker used in the tests.
* ``binding`` -- argument marshalling for the C-ABI library ``libhexdecode.so`` built from
                 ``csrc/``.  Every step of the decode path runs in the HIP kernels behind it.

Importing the package loads nothing native; ``binding.load()`` does, and raises if the
library has not been built (there is no CPU fallback).
"""

__all__ = ["synth", "binding"]
