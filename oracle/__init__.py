"""CPU oracle of the BFP KV-cache path: test infrastructure, never part of the product path."""
