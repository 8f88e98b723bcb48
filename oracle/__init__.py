"""CPU oracle: test infrastructure only (see msrl_ref.c)."""
