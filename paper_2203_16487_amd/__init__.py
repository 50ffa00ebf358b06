"""MI355X-native SpecDec (arXiv 2203.16487) draft-then-verify hot path.

`synth`   : seeded synthetic inputs (NumPy only).
`binding` : ctypes binding of libspecdec.so (the HIP library); imported lazily so
            that `synth` can be used on machines without the built library.
"""
