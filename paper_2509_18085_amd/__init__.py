"""MI355X-native draft-graph verification step of Spiffy (arxiv 2509.18085).

``paper_2509_18085_amd.spiffy``  - thin ctypes binding over the C-ABI HIP library
                                   (loads libspiffy.so; raises if it is not built)
``paper_2509_18085_amd.synth``   - seeded synthetic inputs (no method arithmetic)
``paper_2509_18085_amd.build``   - compiles csrc/*.hip for gfx950 into libspiffy.so

Importing this package loads nothing; import the submodule you need.
"""
__all__ = ["spiffy", "synth", "build"]
