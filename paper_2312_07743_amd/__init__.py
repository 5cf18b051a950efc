"""MI355X-native SGNS (word2vec) training hot path of FULL-W2V.

The product is the C-ABI library built from csrc/ (see include/w2v.h);
`binding` is a thin ctypes layer over it, `synth` makes seeded synthetic corpora."""
