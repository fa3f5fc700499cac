"""CPU oracle for the PipeMare training step.  Test infrastructure only (see pipemare_oracle.py)."""
