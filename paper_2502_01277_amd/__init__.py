"""MI355X-native hot path of a cascaded video-analytics serving pipeline:
ctypes binding over the C-ABI library built from csrc/ (see include/octo.h),
plus the seeded workload generators (zoo, synth) that feed tests and benchmarks.
"""
