"""MI355X (gfx950) implementation of the server-side quasi-Newton step of
Arnold & Wang, "Accelerating SGD for Distributed Deep-Learning Using
Approximated Hessian Matrix" (Section 2, eq. (2)-(4)).

`qn` is a thin binding over the C ABI of libqn.so (include/qn.h, include/qn_diag.h):
it only marshals torch tensors into device pointers (torch also owns the scratch
memory the library's passes use).  `synth` generates the seeded
synthetic worker states.  There is no CPU fallback: every call fails loudly
when the HIP library has not been built.
"""
from . import synth  # noqa: F401
from .qn import (qn_update, qn_update_noalloc, qn_gram, qn_eig, qn_apply, qn_init,  # noqa: F401
                 qn_hinv, qn_gemv_t, qn_coef, qn_hinv_apply,
                 qn_update_bounded, qn_tau_bound, BOUND_SIGMA1, BOUND_SECANT,
                 trace_begin, trace_end, probe_copy, probe_read, probe_chain, diag_gram,
                 workspace_bytes, GramState, GRAM_AUTO, GRAM_STREAM, GRAM_SMALL,
                 KERNEL_NAMES, QnError)
