"""CPU oracle for the Power-SMC step: test infrastructure only (never imported by the product path)."""
