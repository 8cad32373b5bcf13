"""MI355X-native online back-propagation training of the CNN variant of Ciresan et al. (2011).

`synth` draws the seeded synthetic workloads; `binding` is the thin ctypes layer over the
C-ABI library built from `csrc/` (imported lazily so that `synth` works without it).
"""
