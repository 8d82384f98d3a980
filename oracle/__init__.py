"""CPU float64 oracle for the MU NMF iteration.  Test infrastructure only:
nothing on the product path imports this package."""
