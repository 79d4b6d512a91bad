"""CPU oracle (test infrastructure only; see inr_oracle.h)."""
