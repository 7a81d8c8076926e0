"""fp64 CPU oracle of the CCA / CCGQA block.  Test infrastructure only: the
product path (paper_2510_04476_amd) never imports this package."""
