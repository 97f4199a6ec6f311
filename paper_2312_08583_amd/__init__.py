"""W6A16 FP6 (E3M2, 4+2 planes) linear layer for MI355X: Python binding of the HIP library."""
