"""MI355X-native batched token sampling (the sampling step that ends every decode iteration).

The product is the C library ``libsip.so`` (sources in ``csrc/``, boundary in
``include/sip.h``); this package is its thin Python binding."""
from .binding import (SIP_BF16, SIP_F32, SIP_MAX_K_LOGPROBS, SIP_MAX_L, SIP_MAX_SHARDS, SIP_MAX_SLOTS, SIP_MAX_V, ShardTable, SipError, load,
                      sip_probe_read, sip_profile_kernel_events, sip_publish_ids, sip_sample, sip_init, sip_noalloc_scratch_bytes, sip_sample_noalloc, sip_sample_call, sip_sample_sharded, sip_sample_state, sip_state_assign, sip_state_bytes,
                      sip_state_init, sip_status_string, sip_version, sip_wait_ids, sip_workspace_bytes, sip_workspace_bytes_sharded,
                      state_table_views, state_views)

__all__ = ["SIP_BF16", "SIP_F32", "SIP_MAX_K_LOGPROBS", "SIP_MAX_L", "SIP_MAX_SHARDS", "SIP_MAX_SLOTS", "SIP_MAX_V", "ShardTable", "SipError", "load",
           "sip_probe_read", "sip_profile_kernel_events", "sip_publish_ids", "sip_sample", "sip_init", "sip_noalloc_scratch_bytes", "sip_sample_noalloc", "sip_sample_call", "sip_sample_sharded", "sip_sample_state", "sip_state_assign", "sip_state_bytes",
           "sip_state_init", "sip_status_string", "sip_version", "sip_wait_ids", "sip_workspace_bytes", "sip_workspace_bytes_sharded", "state_table_views", "state_views"]
