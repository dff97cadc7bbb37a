"""CPU oracle for the ConvAttn forward pass.  Test infrastructure only."""
