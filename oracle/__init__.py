"""fp64 CPU oracle for the hybrid delta attention path.  TEST INFRASTRUCTURE ONLY:
nothing in the product package may import this."""
