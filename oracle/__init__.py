"""CPU oracle of the LAVa eviction path (test infrastructure; see lava_oracle.py)."""
