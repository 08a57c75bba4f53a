"""MI355X-native hot path of sensitive-sparse zeroth-order fine-tuning.

`synth` holds the seeded input generators (numpy only).  `szo` is the thin
binding over the C-ABI library built from `csrc/`; it is imported lazily so
that the input generators can be used without the native library.
"""
