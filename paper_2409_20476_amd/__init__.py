"""shm355: device-initiated, work-group-collaborative OpenSHMEM data movement on one MI355X.

``paper_2409_20476_amd.shm``   ctypes binding of libshm355.so (the product; needs the built library)
``paper_2409_20476_amd.synth`` seeded input generators (no library needed)
``paper_2409_20476_amd.build`` compiles the library with hipcc for gfx950
"""
