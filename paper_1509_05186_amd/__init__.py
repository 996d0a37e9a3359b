"""E-Tree / E-Forest asymmetric distance computation on MI355X: Python binding of the C ABI.

Argument marshalling only: every step of the computation runs in the HIP library
(``lib/libetf.so``, built by ``paper_1509_05186_amd.build``).  Importing this package
without the built library raises; there is no CPU fallback.
"""
from .binding import (ETF_MODE_FLAT, ETF_MODE_FOREST, ETF_MODE_TREE, ETF_PROBE_COPY, ETF_PROBE_LDS, ETF_PROBE_LDS_SCATTER, ETF_PROBE_READ, ETF_PROBE_ROWS,
                      ETF_PROBE_MFMA_F32, ETF_PROBE_VALU_ADD3, ETF_PROBE_VALU_F32, ETF_PROBE_VALU_PK16,
                      ETF_PROBE_WRITE, Context, EtfError, EtfLayout, EtfStats,
                      library_path, load_library)

__all__ = ["Context", "EtfError", "EtfStats", "EtfLayout", "ETF_MODE_FLAT", "ETF_MODE_TREE", "ETF_MODE_FOREST",
           "library_path", "load_library",
           "ETF_PROBE_READ", "ETF_PROBE_WRITE", "ETF_PROBE_COPY", "ETF_PROBE_ROWS", "ETF_PROBE_LDS", "ETF_PROBE_LDS_SCATTER",
           "ETF_PROBE_VALU_F32", "ETF_PROBE_VALU_ADD3", "ETF_PROBE_VALU_PK16", "ETF_PROBE_MFMA_F32"]
