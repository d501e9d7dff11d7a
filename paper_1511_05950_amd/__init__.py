"""MI355X-native hot path of staleness-aware n-softsync ASGD: HIP kernels behind a C ABI (csrc/,
include/sasgd.h) and a ctypes binding (binding.py).  Nothing is loaded at import time."""
