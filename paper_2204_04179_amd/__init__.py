"""MI355X-native hot path of GRAM (item-deduplicated encode / gradient accumulate).

`paper_2204_04179_amd.gram` is the binding of the C-ABI HIP library;
`paper_2204_04179_amd.workloads` draws the seeded synthetic inputs.  Importing
the package loads nothing: the shared library is opened on first use.
"""
