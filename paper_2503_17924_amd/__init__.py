"""MI355X-native document-masked attention, CP sharding maps and WLB packing.

The Python layer only marshals arguments to the C-ABI library built from
`csrc/` (see `binding.py`); `workloads.py` holds the seeded input generators.
"""
