"""Exact softmax-attention forward/backward for MI355X (gfx950) behind a C ABI.

`attn` is the thin ctypes binding of libattn_mi355x.so (argument marshalling only);
`synth` draws the seeded synthetic inputs.  Nothing here computes attention on the CPU.
"""
