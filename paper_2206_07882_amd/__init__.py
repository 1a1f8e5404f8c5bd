"""INT4 RNN-T inference with density-ratio LM fusion for AMD MI355X (gfx950).

``qrnnt`` is the thin ctypes binding of the C-ABI library ``libqrnnt.so``;
``synth`` draws the seeded synthetic inputs; ``build`` compiles the library.
"""
