"""CPU oracle of the dMath hot path.  Test infrastructure only; see ``cpu_oracle.py``."""
