"""MI355X-native per-token core of Truncated PPO (T-PPO).

``binding`` wraps the C-ABI library (HIP kernels for gfx950); ``synth`` draws
the seeded synthetic workloads.  Importing the package loads neither torch nor
the shared library; ``binding`` does, and fails loudly if the library is
missing.
"""
