"""CPU oracle for the MoE expert layer (test infrastructure, never imported by the product path)."""
