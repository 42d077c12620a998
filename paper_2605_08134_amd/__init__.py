"""MI355X-native DARE attention-layer step: HIP kernels behind a C ABI, with a
thin ctypes binding (``paper_2605_08134_amd.binding``).  Importing the package
loads nothing native; the binding loads ``libdare.so`` on first use and raises
if it has not been built."""
