"""MI355X-native Q-GaLore optimizer step (HIP kernels behind a C ABI).

`paper_2407_08296_amd.qgalore` is the thin ctypes binding of libqgalore.so;
`paper_2407_08296_amd.inputs` holds the seeded synthetic input generators.
Nothing is loaded at package import; the binding loads the shared library on
first use and raises if it has not been built.
"""
