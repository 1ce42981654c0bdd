"""qsv: batched complex64 state-vector simulation of layered circuits for MI355X (gfx950).

``binding`` is the ctypes layer over libqsv.so; ``workloads`` draws the seeded synthetic inputs;
``build`` compiles the library in-tree.  Nothing is loaded at import time.
"""
