"""MI355X-native snapshot path of lazy asynchronous multi-level checkpointing (one GPU's shard).

`binding` loads the HIP library (C-ABI in include/ckpt.h and include/ckpt_proxy.h); `shards`
describes the seeded synthetic workloads. Nothing is imported eagerly: `shards` must stay usable
without the built library."""
