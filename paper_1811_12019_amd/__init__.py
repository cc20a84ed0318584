"""MI355X-native K-FAC hot path (factor build, running average, damped inverse, preconditioning).

The compute lives in the HIP library built from ``csrc/`` and exposed through a C ABI
(``include/kfac.h``); ``binding`` is a thin ctypes layer with the same entry-point names.
"""
