"""MI355X-native executor for one MPMD pipeline stage (see include/jpp.h).

`inputs` holds workload shapes and seeded synthetic data; `binding` is the thin
ctypes layer over the C-ABI library built from csrc/.  Importing the package
does not load the library; calling into `binding` does, and fails loudly if it
has not been built.
"""
