"""CPU oracles (test infrastructure only; the product path never imports this package)."""
