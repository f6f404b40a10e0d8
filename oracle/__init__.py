"""CPU oracle package (test infrastructure; see tlora_oracle.py)."""
