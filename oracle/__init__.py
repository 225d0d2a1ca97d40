"""CPU oracle for the FastMTP draft path.  Test infrastructure only: nothing in the
product package may import this."""
