"""MI355X-native hot path of randomized-partition model-aggregation GNN training.

The compute lives in ``csrc/`` (HIP, gfx950) behind the C ABI declared in
``include/tma.h``; ``binding`` is the argument-marshalling layer over it.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""
__version__ = "0.1.0"
