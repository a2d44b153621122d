"""MI355X-native hot path of collective KV-cache reuse and diff-aware storage.

`paper_2604_03143_amd.tdk` is the thin binding over the C-ABI library
(libtdk.so, hand-written HIP for gfx950); `paper_2604_03143_amd.workload`
builds seeded synthetic rounds.  Nothing is loaded at import time.
"""
