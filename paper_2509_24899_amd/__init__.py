"""MI355X-native hybrid-attention forward (Attention Surgery, arXiv 2509.24899, Sec. 3.2).

`hybrid_attn` holds the ctypes binding over the C-ABI library (loaded on first use, and a loud
error when it is not built); `workloads` holds the seeded synthetic input recipes.
"""
