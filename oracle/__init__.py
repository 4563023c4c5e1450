"""CPU oracle (test infrastructure only; see dllava_ref)."""
