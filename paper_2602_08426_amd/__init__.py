"""MI355X-native hot path of Prism (spectral-aware block-sparse prefill attention).

Importing the package does not load the HIP library; `paper_2602_08426_amd.binding`
loads `libprism.so` on first use and raises if it is missing.
"""
