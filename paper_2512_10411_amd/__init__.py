"""MI355X-native SWA + sink ("keep first k") prefill attention (arXiv 2512.10411).

The compute path is a hand-written HIP kernel for gfx950 behind a C-ABI
library (``libswaa.so``); :mod:`.binding` marshals torch tensors into it and
:mod:`.inputs` makes the seeded synthetic workloads.  Nothing here falls back
to a CPU or PyTorch implementation: a missing library is an error.
"""
__version__ = "0.1.0"
