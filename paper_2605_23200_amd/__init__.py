"""MI355X-native hot path of Adaptive Mass-Segmented (AMS) KV compression.

`paper_2605_23200_amd.binding` is the thin Python face of the C-ABI library
(include/ams.h); `paper_2605_23200_amd.inputs` draws the synthetic caches.
"""
