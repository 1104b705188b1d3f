"""CPU oracle for decode-step MFA: test infrastructure, never part of the product path."""
