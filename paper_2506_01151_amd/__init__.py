"""Python binding of the zapformat HIP library (argument marshalling only)."""
from .binding import (Engine, State, StateBatch, Twin, ZfError, load_library, compile, advance, compute_mask, compute_mask_async, compute_mask_apply_async, compute_mask_noalloc, mask_wait, apply_mask,  # noqa: F401
                      ZF_OK, ZF_ERR_INVALID_ARG, ZF_ERR_GRAMMAR, ZF_ERR_REJECTED, ZF_ERR_RANGE,
                      ZF_ERR_DEVICE, ZF_ERR_OOM, ZF_ERR_OVERFLOW)
