"""CPU oracle for the SparQ decode step.  Test infrastructure only: nothing in the
product package imports this, and this imports nothing from the product package."""
