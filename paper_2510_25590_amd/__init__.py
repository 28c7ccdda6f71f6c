"""RegionE region-aware denoising step for AMD MI355X (gfx950).

`inputs` holds the seeded synthetic input generators; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/`.  Importing the package does not load the
library; the first call into `binding` does, and raises if it has not been built.
"""
