"""SuperKMeans hot path for AMD MI355X (gfx950).

``paper_2603_20009_amd.skm``      thin ctypes binding of the C-ABI library (``libskm.so``)
``paper_2603_20009_amd.datagen``  seeded synthetic inputs

Nothing is loaded at import time; ``skm`` loads the HIP library on first use
and raises if it has not been built.
"""
__all__ = ["skm", "datagen"]
