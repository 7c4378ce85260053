"""MI355X (gfx950) implementation of the Token Filtering hot path: KV-similarity scoring,
variance-aware head fusion, exact-count filtering, compaction and attention over the kept
tokens.  The work is done by hand-written HIP kernels behind a C ABI (include/tokfilt.h);
`binding` marshals arguments to it, `synth` draws seeded inputs, `build` compiles it."""
