"""CPU fp64 oracle (test infrastructure only; the product path never imports this)."""
