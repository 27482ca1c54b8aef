"""MI355X-native direct convolution (forward, backward-by-data, weight update).

``paper_1808_05567_amd.conv`` is the thin binding over the C-ABI HIP library;
``paper_1808_05567_amd.inputs`` holds the seeded synthetic workloads.  Importing
the package loads nothing native; the library is loaded on first use and its
absence is an error, never a fallback.
"""

import os as _os

# Kernel arguments in device memory: a workgroup's first instructions read them, and from host
# memory (the runtime's default placement) that read takes 1 - 3 us for every workgroup; a
# convolution tile lives 7 - 40 us.  Measured over the 20 layers of the benchmark at N = 256:
# +0.8 % (fp32), +2.8 % (bf16).  A setting of the HIP runtime, read when it initialises: it
# takes effect if this package is imported before the first HIP call of the process; an
# explicit setting in the environment wins.
_os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")
