"""MI355X-native attention for one rank of MM-SP (zigzag ring steps + Ulysses head shard)."""
