"""MI355X (gfx950) implementation of EcoSpa's coupled-sparsification hot path.

The work is done by hand-written HIP kernels behind a C ABI (``include/ecospa.h``);
:mod:`.binding` marshals arguments to it.  There is no CPU fallback: loading fails
loudly when the built library is missing.
"""
