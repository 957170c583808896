"""MI355X-native shared-attention (SAN) Transformer decoding.

`binding` wraps the C-ABI library (include/san.h) built from csrc/;
`workloads` draws the seeded synthetic inputs; `build` compiles the library.
"""
