"""MI355X-native dense GEMM (C = A x B) behind a C ABI, with a thin Python binding.

``gemm_f32`` / ``gemm_bf16`` and friends live in :mod:`.fsrgemm` and are
re-exported here; the shared library is loaded on first use and every call
raises if it is absent.  :mod:`.inputs` holds the seeded operand generators.
"""
from .fsrgemm import *  # noqa: F401,F403
from .fsrgemm import __all__  # noqa: F401
