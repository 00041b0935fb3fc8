"""MI355X-native Dynamic SplitFuse attention step (paper: DeepSpeed-FastGen).

``paper_2401_08671_amd.fsf``       ctypes binding of the C-ABI library (HIP kernels + host composer)
``paper_2401_08671_amd.workloads`` seeded synthetic inputs (no method arithmetic)
``paper_2401_08671_amd.build``     hipcc build of the shared library for gfx950

Importing the package loads nothing native; ``fsf`` loads the library on first use and
raises if it has not been built.
"""
