"""MI355X-native optimizer-step hot path for SSD-offloaded mixed-precision fine-tuning.

`paper_2505_23254_amd.binding` is the Python face of the C-ABI library built from `csrc/`
(it raises at import if the library has not been built).  `paper_2505_23254_amd.synth` holds
the seeded synthetic workloads; it contains none of the method's arithmetic.
"""
