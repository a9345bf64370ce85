"""MI355X-native FO-SGD gradient codec (arXiv 2405.11095): Python side.

`binding` marshals arguments into the C-ABI library built from `csrc/`; `inputs` holds the seeded
synthetic gradient generators used by tests and the benchmark.  Importing the package does not
load the HIP library; the first codec call does, and raises if it has not been built.
"""
