"""MI355X-native CP multi-token-prediction head (loss forward/backward and draft sampling).

The compute lives in ``csrc/`` (hand-written HIP for gfx950 behind a C ABI declared in
``include/cp_head.h``); ``binding`` marshals arguments to it and ``synth`` draws seeded inputs.
Importing the package loads nothing native; ``binding.lib()`` does, and fails loudly if the
library has not been built.
"""
