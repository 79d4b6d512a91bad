"""MI355X-native batched decode of INR-compressed image datasets (Rapid-INR decode path).

`rinr` is the thin ctypes binding over the C-ABI library built from `csrc/`;
`synth` is the seeded input generator.  Importing the package does not load the
library; `rinr.lib()` does and raises if it has not been built.
"""
