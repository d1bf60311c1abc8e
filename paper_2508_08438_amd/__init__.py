"""MI355X-native selective-reuse prefill path (visible prefix match, reuse counters,
KV page gather, paged causal GQA prefill attention) behind a C-ABI library.

`inputs` (seeded synthetic workloads) imports without the HIP library; everything in
`binding` needs `libskv.so` and raises if it is not built.
"""
