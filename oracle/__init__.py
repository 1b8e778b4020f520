"""CPU oracle of the BRGEMM hot path.  Test infrastructure: see reference.py."""
