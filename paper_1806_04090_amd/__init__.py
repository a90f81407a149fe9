"""MI355X-native ATOMO gradient encoder/decoder (arXiv 1806.04090): HIP kernels behind a C ABI."""
