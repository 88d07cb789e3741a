"""CPU oracle (test infrastructure only; see decoder.py)."""
