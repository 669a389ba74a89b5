"""CPU oracle (test infrastructure only; the product path never imports this package)."""
