"""CPU oracle for the DDD draft round: test infrastructure only, never imported by the product path."""
