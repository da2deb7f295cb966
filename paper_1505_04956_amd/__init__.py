"""MI355X-native ASGD mini-batch K-Means: C-ABI HIP library plus a thin ctypes binding."""
