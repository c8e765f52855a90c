"""libkvra: KV-Runahead's per-chunk prefill hot path (RoPE + KV append, chunked causal attention,
context-level load balancing) written in HIP for gfx950.  `kvra` is the ctypes binding of the
C-ABI library, `synth` the seeded input generators, `build` compiles the library in-tree."""
