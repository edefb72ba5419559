"""CPU oracle of the XNOR-Net forward binary convolution.  TEST INFRASTRUCTURE ONLY:
imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg, never
by the product path (paper_1603_05279_amd)."""
