"""CPU oracle of the MoE-layer hot path.  Test infrastructure only: the product never imports it."""
