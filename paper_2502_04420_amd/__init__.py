"""MI355X-native mixed-precision KV-cache quantization and fused decode attention.

The work is done by hand-written HIP kernels behind the C ABI of ``include/kvq.h``
(built into ``libkvq.so`` by ``paper_2502_04420_amd.build``); this package is the thin
Python binding with the same call names.  There is no CPU fallback: using the binding
without the built library raises.
"""
from .binding import (KEYS_PER_CHANNEL, KEYS_PER_TOKEN, KVQ, KVQError, META_FP16, META_FP32, library_path,  # noqa: F401
                      load_library)
from .schedule import equivalent_precision, bytes_per_token, parse_pairs  # noqa: F401
