"""MI355X-native paged attention (batched decode + chunked prefill) over an extensible KV pool.

`paper_2412_18169_amd.kun` is the thin ctypes binding of the C-ABI library (include/kun.h);
`paper_2412_18169_amd.synth` generates the seeded synthetic workloads.  Neither is imported here,
so that the input generator can be used on machines without the built library.
"""
