"""CPU oracle for the KSA hot path.  Test infrastructure only: nothing in the
product package may import this."""
