"""CPU oracle for the Gibbs sweep.  TEST INFRASTRUCTURE: not part of the product path."""
