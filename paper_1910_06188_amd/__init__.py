"""MI355X-native int8 quantized fully-connected layer (Q8BERT inference hot path).

`paper_1910_06188_amd.q8` is the binding over the C-ABI library built from csrc/;
`paper_1910_06188_amd.synth` holds the seeded input generators.  Importing the package
itself loads nothing, importing `q8` fails loudly if the HIP library is not built.
"""
__version__ = "0.1.0"
