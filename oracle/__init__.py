"""CPU oracles (test infrastructure only; the product package never imports this)."""
