"""CPU checker for the Global Resolution verifier (test infrastructure, never imported by
the product path)."""
