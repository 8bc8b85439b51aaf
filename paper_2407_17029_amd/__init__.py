"""MI355X-native adapted quantized linear layer (Q-BLoRA / QA-BLoRA hot path).

`paper_2407_17029_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`; `paper_2407_17029_amd.synth` draws the seeded synthetic
workloads.  Nothing is loaded at import time; the binding raises if the HIP
library has not been built.
"""
