"""CPU oracle for the FourierAttention hot path (test infrastructure only).

Everything under this package is a slow, definitional fp64 implementation of
what `fa_compress` and `fa_decode` compute, written from the paper's
Section 3.3 (Eq. 1-6).  It exists so that the HIP kernels can be checked
against something that is not themselves.

Rules this package obeys:
  * it imports nothing from the product package and shares no code, tables or
    constants with the HIP path;
  * only tests, the smoke check and the CPU-baseline leg of the benchmark may
    import it; the product never routes through it;
  * no blocking, fusion or algebraic reordering beyond what the paper's
    equations state (the basis matrix, the reconstructed K/V and the softmax
    are all materialised explicitly).
"""

from .legt import (  # noqa: F401
    legt_positions,
    legt_basis,
    legt_weights,
    legt_compress,
    legt_reconstruct,
    legt_mse,
)
from .fourier_kv import (  # noqa: F401
    basis_matrix,
    basis_weights,
    compress_segment,
    reconstruct_segment,
    attend,
    decode_head_group,
    compress_batched,
    decode_batched,
)
