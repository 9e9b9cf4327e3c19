"""MI355X-native blocked sparse x dense multiply (1-SA reordering, VBR, MFMA SpMM).

``binding``  ctypes front of the C-ABI library (``include/vbr_spmm.h``); importing it requires the
             built ``libvbr_spmm.so`` -- there is no fallback path.
``synth``    seeded synthetic inputs (no method arithmetic).
``build``    in-tree hipcc build of the library.
"""
