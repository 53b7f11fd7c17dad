"""MI355X-native hot path of Sufficient Factor Broadcasting: a thin Python binding over
libsfb.so (hand-written HIP kernels behind a C ABI, declared in include/sfb.h).

Importing this package loads the compiled library and raises ImportError if it has not
been built (python paper_1511_08486_amd/build.py, or __graft_entry__.build()).  There
is no CPU fallback.
"""
from .binding import (  # noqa: F401
    SFB_MLR, SFB_DML, SFB_L2SVM, SFB_F32, SFB_BF16, SfbError, SfbBatch, Sfb, SspSimulator, halton_receivers, lib, library_path,
    sfb_strerror,
)
