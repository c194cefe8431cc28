"""MI355X-native 4D FNO spectral convolution / FNO block (HIP kernels behind a C ABI).

The binding in .binding loads libfno.so lazily on first use and raises if it is missing;
there is no CPU fallback.  synth holds the seeded input generators only.
"""
