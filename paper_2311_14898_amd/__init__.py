"""MI355X-native hot path of partition-based full-graph GCN training.

The compute lives in the HIP library built from csrc/ (see include/hongtu.h);
`binding` marshals arguments into it and nothing else.  Importing this package
does not load the library; `binding.load()` does and fails loudly if it is
missing.
"""
