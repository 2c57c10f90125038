"""libadapshot: MI355X-native hot path of AdapShot's KV-cache reuse (gather, RoPE re-encode,
query-over-cache attention, probe entropy).  The HIP library is loaded lazily by `binding`."""
