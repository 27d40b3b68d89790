"""MI355X-native hot path of Quantized Optimistic Dual Averaging (arXiv 2505.14371).

``paper_2505_14371_amd.qoda``      thin ctypes binding over the C-ABI library (include/qoda.h)
``paper_2505_14371_amd.workloads`` seeded synthetic inputs (no arithmetic of the method)
``paper_2505_14371_amd.build``     compiles csrc/*.hip for gfx950 into libqoda.so next to this file

Importing the package loads nothing; the library is opened on first use and its absence is an error.
"""
