"""CPU oracle for the DGS hot path.  Test infrastructure only: nothing in the
product package imports this."""
