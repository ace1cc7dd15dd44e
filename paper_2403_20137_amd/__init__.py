"""BFP KV cache with offline channel reordering on MI355X (gfx950): Python binding of libkvbfp."""
