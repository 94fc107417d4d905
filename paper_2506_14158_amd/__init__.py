"""MI355X-native tree-verification step (tree-masked attention, path acceptance, KV compaction)."""
