"""MI355X-native online path of Squeezed Attention: centroid scoring, threshold selection with
key-range compaction, sparse flash attention (decode and prefill) and the two-level lookup.

`binding` wraps the C-ABI library built from `csrc/`; `workload` draws the seeded synthetic inputs.
"""
