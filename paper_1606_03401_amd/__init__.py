"""Memory-efficient LSTM back-propagation through time for AMD MI355X (gfx950).

The product is the C-ABI library built from ``csrc/`` (declared in ``include/mebptt.h``);
``binding`` is a thin ctypes layer with the same entry points and ``workloads`` holds the
seeded synthetic input generators.  Importing the package does not load the library; the first
call into ``binding`` does, and fails loudly if it has not been built.
"""
