"""CPU oracle of the Kimad+ compression step.  Test infrastructure only: see kimad_oracle.py."""
