"""MI355X-native Plan-Verify-Fill decoding round: hand-written HIP kernels behind a C ABI
(include/pvf.h) plus this thin ctypes binding.  Build with `python -m paper_2601_12247_amd.build`."""
from . import binding  # noqa: F401
