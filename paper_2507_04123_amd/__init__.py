"""MI355X-native hot path of the EMC2 LiDAR branch: voxelize -> kernel map -> sparse conv -> project/gather.

The compute lives in the HIP library under ``csrc/`` (C-ABI declared in ``include/emc2.h``);
``binding`` is the thin ctypes layer over it.  ``configs`` and ``gen`` hold only workload shapes and
seeded input generators.
"""
