"""MI355X-native per-layer query-centric KV-cache fusion (rerope, score, select,
recompute_qkv, scatter, recompute_attn) behind a C-ABI library.

`inputs` holds the seeded workload generators; `binding` loads the HIP library
lazily and fails loudly when it is missing.
"""
