"""CPU oracle for PASA attention forward.  Test infrastructure only: see pasa_oracle.py."""
