"""MI355X-native HARP structured-rotation library: HIP kernels behind a C ABI (csrc/),
a ctypes binding (harp.py) and seeded synthetic inputs (inputs.py).

Nothing is imported eagerly: ``from paper_2605_29843_amd import harp`` loads the HIP
shared library and raises if it has not been built.
"""
__version__ = "0.1.0"
