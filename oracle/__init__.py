"""CPU oracle of the VMoBA hot path.  Test infrastructure only: see vmoba_oracle.py."""
