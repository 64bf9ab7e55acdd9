"""CPU oracle for KV block rotation: test infrastructure, never the product path."""
