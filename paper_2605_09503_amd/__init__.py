"""MI355X-native per-group-quantized linear layer (PermuQuant hot path).

`paper_2605_09503_amd.pq` is the thin binding over the C-ABI library built from csrc/;
`paper_2605_09503_amd.synth` draws the seeded synthetic inputs.  Importing this package
does not load the GPU library; the binding loads it on first use and raises if it is missing.
"""
