"""MI355X-native swap-aware training iteration (layer-pack-major, Harmony, arxiv 2202.01306).

`binding`  ctypes binding of the C-ABI library libhmy.so (built by `build.py`)
`synth`    seeded synthetic inputs (no arithmetic of the method)
"""
