"""MI355X-native paged KV-cache data path: paged decode attention and KV-block pack/restore."""
