"""CPU oracle of the decode path.  Test infrastructure only: see absb_oracle.c."""
