"""CPU oracle for the AED decoder step (test infrastructure; see aed_oracle.h)."""
