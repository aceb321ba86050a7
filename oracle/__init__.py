"""CPU oracle of the DEF / DEF-A step (arXiv 2004.05298).  Test infrastructure:
imported by tests, the smoke check and the benchmark's CPU-baseline leg only."""
