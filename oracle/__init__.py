"""CPU checker package (test infrastructure; never imported by the product)."""
