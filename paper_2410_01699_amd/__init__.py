"""MI355X-native hot path of Speculative Jacobi Decoding (window forward + probabilistic
verification) behind a C-ABI library.  `synth` holds the seeded input generators; `binding`
loads the HIP library and raises if it is not built."""
