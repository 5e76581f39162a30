"""CPU oracle (test infrastructure): see ivfadcr_oracle.py."""
