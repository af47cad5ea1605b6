"""MI355X-native Vamana beamSearch / batch insertion / RaBitQ (libjx).

Submodules:
  datagen -- seeded synthetic workloads (importable without a GPU)
  jx      -- ctypes binding of the HIP library; importing it raises if
             libjx.so has not been built (there is no CPU fallback)
  build   -- compiles libjx.so in-tree with hipcc for gfx950
"""
