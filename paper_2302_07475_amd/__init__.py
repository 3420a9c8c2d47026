"""MI355X-native hot path of S3GD-MV (sparse sign SGD with majority vote).

`paper_2302_07475_amd.s3gd` is the ctypes binding of the C-ABI library built
from `csrc/`; `paper_2302_07475_amd.datagen` holds the seeded input recipes.
Nothing is imported eagerly so that the input generators stay usable on a
machine without the built library.
"""
