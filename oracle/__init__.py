"""CPU oracle of the MuKV hot path -- test infrastructure only (see oracle.py)."""
