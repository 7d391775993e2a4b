"""MI355X-native speech augmentation + power-mel front end (HIP kernels behind a C ABI)."""
__version__ = "0.1.0"
