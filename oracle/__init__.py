"""CPU oracle for the FAVOR# hot path.  Test infrastructure only: nothing in the
product package imports this."""
