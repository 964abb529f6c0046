"""MI355X-native CafeQ hot path: HIP kernels behind a C-ABI library, with a thin
ctypes binding (``paper_2511_19705_amd.cafeq``).  Importing the package does not
load the library; ``cafeq`` does, and fails loudly when it has not been built."""
