"""Lossless decompression of compressed bf16 MoE expert weights on MI355X.

``paper_2601_21198_amd.zipmoe`` is the binding of the C-ABI library;
``paper_2601_21198_amd.synth`` holds the seeded synthetic inputs.  Nothing is
imported eagerly, so the input generators can be used without the library.
"""
