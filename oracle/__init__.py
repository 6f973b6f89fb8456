"""CPU oracle for the GXPO update engine.  Test infrastructure only."""
