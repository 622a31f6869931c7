"""Subsampled Gauss-Newton path for fully-connected networks on MI355X (libdn + thin binding)."""
from .binding import (  # noqa: F401
    DN_FULL, DN_BLOCKDIAG, DN_PARTITION, DnError, Context, lib_path, load_library,
    dn_forward, dn_forward_static, STATIC_SCRATCH_BYTES, dn_grad, dn_jacobian_prep, dn_jacobian_read, dn_gn_matvec, dn_gn_matvec_rop, dn_cg, dn_cg_sync, dn_newton_step,
    NewtonParams, NewtonStats,
)
