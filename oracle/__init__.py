"""CPU oracle of the HiRE decode-step path (test infrastructure only; see hire_oracle.c)."""
