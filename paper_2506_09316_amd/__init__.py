"""MI355X-native dual-state linear attention (DSLA) layer forward.

The compute lives in a C-ABI shared library built from csrc/ (hand-written gfx950 HIP
kernels); `binding` is a thin ctypes layer with the same entry-point names.  Importing
the package does not load the library; the first call does, and fails loudly if the
library has not been built.
"""
from .binding import (dsla_project, dsla_attention_prefill, dsla_conversion_plan, dsla_kv_cache_bytes, dsla_max_conversion_rate, dsla_rank_layers,  # noqa: F401
                     )
from .binding import (DslaDesc, DslaError, DslaMulti, dsla_decode_multi, dsla_prefill_multi,  # noqa: F401
                      dsla_prefill_multi_workspace_bytes, make_multi,  # noqa: F401
                      dsla_attention_decode, dsla_attention_decode_workspace_bytes,  # noqa: F401
                      dsla_attention_entropy, dsla_attention_entropy_workspace_bytes,  # noqa: F401
                      dsla_decode, dsla_decode_slots, dsla_prefill, dsla_prefill_static_ws,  # noqa: F401
                      dsla_prefill_varlen, dsla_prefill_varlen_workspace_bytes, dsla_prefill_workspace_bytes,
                      dsla_state_init, library_path, load_library, make_desc, profile_collect, profile_enable)
