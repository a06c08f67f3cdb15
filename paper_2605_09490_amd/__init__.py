"""tkv: tiered KV-cache decode attention for MI355X (gfx950) -- Python face of the C-ABI library libtkv.so."""
from .binding import (LIB_PATH, SYMBOLS, TieredKV, TkvError, load_library, probe_hbm_read, tier_counts,  # noqa: F401
                      TKV_OK, TKV_EINVAL, TKV_ENOMEM, TKV_ECAPACITY, TKV_ESTATE, TKV_EDEVICE)
