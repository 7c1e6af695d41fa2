"""Choreographed attention for AMD MI355X (gfx950): a C-ABI library (libpc.so,
declared in include/pc.h) plus this thin ctypes binding."""
from .binding import (  # noqa: F401
    PC_BF16, PC_F32, PC_FLAG_GROW_EXTENTS, PC_FLAG_HOST_ONLY, PC_OK, PC_POS_AUTO, PC_SLOT_ALIGN,
    PC_ERR_BAD_MSG_ID, PC_ERR_HIP, PC_ERR_INVALID_ARG, PC_ERR_NO_SPACE, PC_ERR_SHAPE,
    Cache, PcError, lib, marshal_calls,
)
