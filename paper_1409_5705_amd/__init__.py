"""MI355X-native sufficient-factor hot path (libsfb) and its thin Python binding."""
from .binding import (  # noqa: F401
    SFB_BF16, SFB_DML, SFB_EHIP, SFB_EINVAL, SFB_ENOWS, SFB_ETOOBIG, SFB_STATIC_SCRATCH_BYTES, SFB_F32, SFB_MLR, SFB_OK, SFB_PROX_NORMALIZE,
    SFB_PROX_PROJECT, SFB_SC, Context, SfbError, SspClock, lib, sfb_batch, strerror, version,
)
