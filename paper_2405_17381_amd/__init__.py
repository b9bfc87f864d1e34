"""MI355X-native Lightning Attention (tiled causal linear attention with decay).

`binding` is the thin ctypes layer over the C-ABI library built from `csrc/`;
`synth` draws the seeded synthetic workloads.  Nothing here computes the
method on the CPU: without the built HIP library the product path raises.
"""
