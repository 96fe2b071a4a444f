"""CPU oracle for the shard forward pass.  Test infrastructure: not part of the product path."""
