"""MI355X-native Q-GenX hot path (quantise, code, decode, average, extra-gradient).

``paper_2308_09187_amd.qgx`` is the thin binding over the C-ABI library built from
``csrc/``; ``paper_2308_09187_amd.synth`` holds the seeded synthetic inputs.
Nothing is loaded at import time; the binding raises if the HIP library is missing.
"""
