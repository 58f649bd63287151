"""One Chimera pipeline worker on one MI355X: C-ABI library (csrc/, built into
libchimera.so), its ctypes binding (binding.py) and the seeded synthetic
workloads (synth.py).  Nothing is loaded at import time."""
