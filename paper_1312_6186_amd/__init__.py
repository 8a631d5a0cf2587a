"""MI355X-native hot path of GPU A-SGD (arXiv 1312.6186).

``paper_1312_6186_amd.binding`` wraps the C-ABI library built from ``csrc/``;
``paper_1312_6186_amd.workloads`` holds the seeded synthetic inputs.  Importing
the package loads nothing; the HIP library is opened on first use and its
absence is an error, never a fallback.
"""
