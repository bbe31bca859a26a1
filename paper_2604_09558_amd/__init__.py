"""Virtual-tensor consumer kernels for MI355X: Python binding over the C-ABI library.

The hot path lives in csrc/ (HIP, gfx950) behind include/vt.h; this package only marshals
arguments.  See build.py for how libvt.so is compiled.
"""
from .binding import *  # noqa: F401,F403
from .binding import (Desc, VtError, build_chain, build_raw, lib, make_op, make_source,  # noqa: F401
                      vt_copy_op, vt_decode_attn, vt_decode_attn_workspace, vt_decode_attn_workspace_init, vt_elementwise, vt_gemm,
                      vt_materialize)
