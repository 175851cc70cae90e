"""MI355X-native verification step of SSSD (arXiv 2411.05894): a C-ABI library of
hand-written HIP kernels (csrc/, built to libsssd_verify.so) and its thin ctypes
binding.  Importing the package does not load the library; calling into it does,
and fails loudly if it was not built."""
