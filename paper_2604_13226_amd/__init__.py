"""KV Packet serving hot path for MI355X: packet store, assembly (RoPE realignment +
concatenation) and query-prefill attention behind the C ABI of include/kvp.h."""
from .binding import *  # noqa: F401,F403
from .binding import load, Store, Cache, KvpError, alloc_workspace, packet_bytes  # noqa: F401
