"""MI355X-native VGG19 forward pass and training step (HIP kernels behind a
C-ABI library, with a thin ctypes binding).  Importing the package is cheap;
the shared library is loaded on first use of :mod:`.binding` and a missing
library is an error, never a fallback."""
