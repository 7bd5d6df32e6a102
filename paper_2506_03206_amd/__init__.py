"""MI355X-native Redistributing Drafter Kernels (RDK): redistribution of a pruned drafter's
distribution onto the target vocabulary and speculative-decoding verification, as a C-ABI HIP
library (``csrc/``) with a thin ctypes binding (``rdk``).  Importing this package loads nothing;
``paper_2506_03206_amd.rdk`` loads the compiled library and fails loudly when it is missing."""
__all__ = ["rdk", "synth"]
