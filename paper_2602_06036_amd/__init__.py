"""MI355X-native DFlash speculative-decoding step: HIP kernels behind a C ABI (include/dflash.h)
plus a thin ctypes binding.  There is no CPU fallback: importing `binding` and calling into it
requires the built library libdflash.so."""
from . import binding  # noqa: F401
from .binding import (Engine, DFlashError, dflash_draft_block, dflash_verify, dflash_accept,  # noqa: F401
                      dflash_kv_commit, dflash_prefill, dflash_kv_read, dflash_kv_write)
