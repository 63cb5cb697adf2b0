"""CPU checker for the LSM key index (test infrastructure, not part of the product)."""
