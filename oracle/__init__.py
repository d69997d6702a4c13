"""CPU oracle of the decoder-stage forward/backward.  TEST INFRASTRUCTURE ONLY: nothing in the product
path may import it; it shares no code with the HIP library."""
