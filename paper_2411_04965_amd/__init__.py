"""MI355X-native quantized linear layers of BitNet a4.8 (HIP kernels behind a C ABI).

Importing the package does not load the native library; the first call into
`paper_2411_04965_amd.binding` does, and raises if it has not been built.
"""
