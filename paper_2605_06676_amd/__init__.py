"""MI355X-native implementation of the LKV inference-time eviction hot path.

``paper_2605_06676_amd.lkv`` is the thin Python binding over the C-ABI library
built from ``csrc/`` (it is loaded on first use and fails loudly when the
library is missing); ``paper_2605_06676_amd.workloads`` draws the seeded
synthetic inputs.  Importing the package itself loads nothing.
"""
