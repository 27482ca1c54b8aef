"""MI355X-native direct convolution (forward, backward-by-data, weight update).

``paper_1808_05567_amd.conv`` is the thin binding over the C-ABI HIP library;
``paper_1808_05567_amd.inputs`` holds the seeded synthetic workloads.  Importing
the package loads nothing native; the library is loaded on first use and its
absence is an error, never a fallback.
"""
