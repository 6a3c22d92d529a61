"""MI355X (gfx950) Online Quantized Memory: the storage / retrieval hot path of
StreamingTOM (arxiv 2510.18269) as hand-written HIP kernels behind a C ABI.

    from paper_2510_18269_amd import oqm      # ctypes binding of libtom_oqm.so

`oqm` raises ImportError if the library has not been built
(python -m paper_2510_18269_amd.build); there is no CPU fallback.
"""
