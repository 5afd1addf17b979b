"""fp64 CPU oracle of the MBConv training step.  Test infrastructure only."""
