"""CPU oracle for the CLaSp hot path -- test infrastructure only (see clasp_oracle.c / clasp_oracle.py)."""
