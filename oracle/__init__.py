"""CPU oracle: test infrastructure only.  The product path never imports this package."""
