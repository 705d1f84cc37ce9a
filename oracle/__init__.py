"""CPU oracle for decentralized neighbor averaging (TEST INFRASTRUCTURE ONLY).

This package is a plain, slow, fp64 numpy statement of what the GPU library
computes: the partial-averaging step of decentralized SGD (eq. dsgd-2), its
fusion with the local update (eqs. dsgd-1, eq.awc, eq.atc, dgd-1/dgd-2), the
synchronous push-sum recursion (section "Asynchronous push-style partial
averaging", with unit delays) and a heavy-ball momentum variant.

It exists so that tests, the smoke check and the benchmark's CPU-baseline leg
have something independent to compare the HIP kernels against.  Nothing in the
product package imports it, and it imports nothing from the product package:
the two share no topology code, no tables and no arithmetic.

Weight matrices are kept as a dictionary of in-neighbor lists,
``W[i] = [(j, w_ij), ...]``, where ``w_ij`` scales the copy of ``x_j`` that
flows from agent ``j`` to agent ``i`` (the index convention of eq. wij).
"""

from . import topology, iterations  # noqa: F401
