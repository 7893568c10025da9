"""CPU oracle of the DLRM-class forward pass.  Test infrastructure only."""
