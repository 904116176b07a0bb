"""MatMulScan prefix sums for MI355X (gfx950).  The binding lives in ``tcuscan``."""
