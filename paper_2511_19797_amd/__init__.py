"""MI355X-native fused attention with a JVP tangent and its backward (see include/tvmattn.h).

The Python layer is a ctypes binding with the C entry points' names; importing the
package does not load the shared library, calling any entry point does (and raises if
it has not been built).
"""
from .binding import (TvmattnError, tvmattn_adaln_jvp_bwd, tvmattn_adaln_jvp_fwd, tvmattn_desc, tvmattn_gate_jvp_bwd, tvmattn_gate_jvp_fwd, tvmattn_gelu_jvp_bwd, tvmattn_gelu_jvp_fwd, tvmattn_jvp_bwd, tvmattn_jvp_bwd_workspace_bytes,  # noqa: F401
                      tvmattn_jvp_bwd_qknorm, tvmattn_jvp_bwd_qknorm_workspace_bytes, tvmattn_jvp_fwd,
                      tvmattn_qknorm_jvp_bwd, tvmattn_qknorm_jvp_bwd_workspace_bytes,
                      tvmattn_qknorm_jvp_fwd, tvmattn_jvp_fwd_qknorm, tvmattn_strerror, tvmattn_jvp_bwd_static, tvmattn_linear_jvp_fwd, tvmattn_linear_jvp_bwd,
                      tvmattn_linear_jvp_bwd_workspace_bytes, TVMATTN_FLAG_PLAIN_ALU,
                      TVMATTN_STATIC_MAX_ROWS,
                      tvmattn_version)
