"""MI355X-native block-sparse attention over a demonstration KV cache (DBSA).

``synth`` holds the seeded input generators; ``binding`` is the ctypes layer
over the C-ABI library ``libdbsa.so`` built from ``csrc/``.  Importing the
package does not load the library; ``binding.lib()`` does, and raises if it
has not been built.
"""
