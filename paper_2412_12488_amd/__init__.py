"""MI355X-native paged KV-cache hot path (prefix-prefill attention, KV append,
page-range pack/unpack) behind a C ABI; this package is its thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, LIB_PATH, McError, lib, mc_pool_desc, pool_desc,  # noqa: F401
                      status_string)
