"""MI355X-native forward hot path of a LocMoE mixture-of-experts layer.

``paper_2401_13920_amd.locmoe`` is the thin binding over the C-ABI library
(``csrc/liblocmoe.so``, hand-written gfx950 HIP kernels); ``workloads`` holds the
seeded synthetic input generators.  Importing the package loads nothing native;
``locmoe.lib()`` loads the shared library and fails loudly if it is not built.
"""
