"""CPU oracle for the MoE dispatch/combine shuffle.  Test infrastructure only."""
