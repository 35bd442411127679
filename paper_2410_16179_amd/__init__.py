"""MI355X-native LSH-sampled decode attention (MagicPIG, arXiv 2410.16179).

`binding` wraps the C ABI of libmagicpig.so (hand-written HIP for gfx950);
`workloads` draws the seeded synthetic inputs; `build` compiles the library in-tree.
"""
