"""CPU oracle for the TEAL decode path. Test infrastructure only (see teal_oracle.c)."""
