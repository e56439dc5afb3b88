"""CPU oracle (plain C + numpy) for the encrypted ternary matmul path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library and its Python binding never
import it, and it never imports them.
"""
from .params import Params  # noqa: F401
from .ckks import Oracle, Ciphertext  # noqa: F401
