"""CPU oracle (test infrastructure). See pdadmm_oracle.py."""
