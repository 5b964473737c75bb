"""CPU oracle for IVF-PQ search: test infrastructure, never a product path."""
