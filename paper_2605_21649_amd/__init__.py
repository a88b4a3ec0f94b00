"""MI355X-native decode hot path of EntmaxKV (sparse alpha-entmax attention over a paged KV cache).

`paper_2605_21649_amd.binding` is the ctypes binding over the C-ABI library (include/entmaxkv.h);
`paper_2605_21649_amd.synth` generates the seeded synthetic workloads.  Importing the package does
not load the HIP library; the first call through the binding does, and raises if it is missing."""
