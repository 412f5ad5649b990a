"""MI355X-native guided source separation hot path (cACGMM EM + mask-based MVDR + STFT/iSTFT).

The compute lives in hand-written HIP kernels behind the C-ABI library `libgss.so`
(see include/gss.h); `binding` is the thin ctypes layer over it and `synth` draws the
seeded synthetic inputs.  Importing this package does not load the library.
"""
