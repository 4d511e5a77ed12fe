"""MI355X-native hot path of variance-based gradient compression.

`paper_1802_06058_amd.vgc` is the ctypes binding of the C-ABI library (loaded on first
use; it raises if the library has not been built).  `paper_1802_06058_amd.workloads`
holds the seeded synthetic inputs.
"""
