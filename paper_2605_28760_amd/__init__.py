"""MI355X-native candidate-state evaluation for Inference-Native ZO.

The product is the C-ABI library built from ``csrc/`` (declared in
``include/zo.h``); ``binding`` marshals arguments to it and nothing else.
``workloads`` holds the seeded synthetic input generators (no arithmetic of the
method).  Importing this package loads nothing; ``binding.lib()`` loads the
shared library and fails loudly when it is missing.
"""
