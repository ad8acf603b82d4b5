"""CPU oracle (test infrastructure only) — see lychee_oracle.c / lychee_oracle.py."""
