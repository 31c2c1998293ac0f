"""MI355X-native Video Sparse Attention hot path (hand-written HIP behind a C ABI).

`paper_2505_13389_amd.vsa` is the thin binding over libvsa.so; `paper_2505_13389_amd.synth`
holds the seeded input generators.  Importing the package loads nothing native.
"""
