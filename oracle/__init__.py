"""CPU oracle for the SRM decode path.  Test infrastructure only: see srm_oracle.c."""
