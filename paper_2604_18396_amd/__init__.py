"""MI355X-native early-exit decode (KV-Shared Exit River) -- Python binding over the C-ABI library."""
