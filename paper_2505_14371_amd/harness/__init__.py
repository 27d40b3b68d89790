"""Measurement harness around the library (no part of the method, nothing the product path imports): the torch-free
probe that profilers and hardware counters are run on, the script that turns their CSV output into the short summaries
under profiles/, and the comparison of layer-wise against global quantization on the same kernels."""
