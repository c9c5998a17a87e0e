"""CPU oracle (test infrastructure only).  Nothing in the product path may import it."""
