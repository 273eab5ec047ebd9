"""MI355X-native Hybrid Target Attention (grouped-query, jagged) behind a C ABI.

``paper_2602_11235_amd.hta`` is the thin Python binding of ``libmtfm_hta.so``;
``paper_2602_11235_amd.inputs`` draws the seeded synthetic workloads.  Nothing here imports
the CPU oracle, and nothing falls back to a CPU path.
"""
